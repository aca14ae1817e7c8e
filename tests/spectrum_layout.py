"""Stored-bin order of a workspace slot, written from include/fftconv.h (test helper)."""
import numpy as np


def stored_bins(N):
    """Arrays (ky, kx) of the B = N*N/2 + 2 stored bins, in storage order."""
    ky = [0] * (N // 2 + 1) + [N // 2] * (N // 2 + 1)
    kx = list(range(N // 2 + 1)) * 2
    for r in range(1, N // 2):
        ky += [r] * N
        kx += list(range(N))
    ky, kx = np.array(ky), np.array(kx)
    assert len(ky) == N * N // 2 + 2
    return ky, kx


def reference_spectrum(maps, N):
    """fp64 spectrum of zero-padded maps [M, e, e] in slot layout [B, M] (complex128)."""
    M, e, _ = maps.shape
    pad = np.zeros((M, N, N))
    pad[:, :e, :e] = maps
    ky, kx = stored_bins(N)
    return np.fft.fft2(pad)[:, ky, kx].T
