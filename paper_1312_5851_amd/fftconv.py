"""ctypes binding of libfftconv.so (declared in include/fftconv.h).

Argument marshalling only: tensors are passed as device pointers, the current
torch stream as a hipStream_t.  Every step of the path runs in the library's
kernels.  Importing this module raises if the library has not been built
(``python -m paper_1312_5851_amd.build`` or ``__graft_entry__.build()``):
there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch  # noqa: F401  (loads the HIP runtime the library binds to)

from . import build as _build

FFTCONV_OK = 0
SPEC_X, SPEC_W, SPEC_G, SPEC_OUT, SPEC_G2 = 1, 2, 4, 8, 16
FPROP, BPROP, ACCGRAD = 0, 1, 2
STATIC_SCRATCH_BYTES = 32 << 20   # workspace limit of fftconv_pass_static
RECOMPUTE = 1   # plan flag: memory-efficient mode (no spectral cache, three-slot workspace)
TRUE_CONV = 2   # plan flag: true convolution (kernel index reversed) instead of cross-correlation
NUM_STAGES = 9
PROFILE_ALL = 0x1FF
STAGE_NAMES = ("fft_x", "fft_w", "fft_g", "cgemm_fprop", "cgemm_bprop", "cgemm_accgrad",
               "ifft_y", "ifft_dx", "ifft_dw")

EXPORTS = (
    "fftconv_plan", "fftconv_plan2d", "fftconv_plan_destroy", "fftconv_fft_size", "fftconv_num_bins",
    "fftconv_workspace_bytes", "fftconv_slot_offset", "fftconv_slot_maps", "fftconv_invalidate",
    "fftconv_valid_slots", "fftconv_fprop", "fftconv_bprop", "fftconv_accgrad", "fftconv_pass_static",
    "fftconv_forward_transform", "fftconv_contract", "fftconv_inverse_transform",
    "fftconv_profile_enable", "fftconv_profile_read", "fftconv_strerror",
    "fftconv_paper_ram_bytes", "fftconv_contraction_flops", "fftconv_tiling",
)


class Desc(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int), ("f", ctypes.c_int), ("fo", ctypes.c_int),
                ("n", ctypes.c_int), ("k", ctypes.c_int), ("flags", ctypes.c_uint)]


class Desc2d(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int), ("f", ctypes.c_int), ("fo", ctypes.c_int),
                ("nh", ctypes.c_int), ("nw", ctypes.c_int), ("kh", ctypes.c_int), ("kw", ctypes.c_int),
                ("flags", ctypes.c_uint)]


class FftconvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


def _load() -> ctypes.CDLL:
    path = _build.lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_1312_5851_amd.build`")
    lib = ctypes.CDLL(path)
    vp, ip, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    sig = {
        "fftconv_plan": (ip, [ctypes.POINTER(vp), ctypes.POINTER(Desc)]),
        "fftconv_plan2d": (ip, [ctypes.POINTER(vp), ctypes.POINTER(Desc2d)]),
        "fftconv_plan_destroy": (ip, [vp]),
        "fftconv_fft_size": (ip, [vp]),
        "fftconv_num_bins": (ip, [vp]),
        "fftconv_workspace_bytes": (sz, [vp]),
        "fftconv_slot_offset": (sz, [vp, ip]),
        "fftconv_slot_maps": (ctypes.c_long, [vp, ip]),
        "fftconv_invalidate": (ip, [vp, ctypes.c_uint]),
        "fftconv_valid_slots": (ctypes.c_uint, [vp]),
        "fftconv_fprop": (ip, [vp, vp, vp, vp, vp, vp]),
        "fftconv_bprop": (ip, [vp, vp, vp, vp, vp, vp]),
        "fftconv_accgrad": (ip, [vp, vp, vp, vp, vp, vp, ip]),
        "fftconv_pass_static": (ip, [vp, ip, vp, vp, vp, vp, ip]),
        "fftconv_forward_transform": (ip, [vp, ip, vp, vp, vp]),
        "fftconv_contract": (ip, [vp, ip, vp, vp]),
        "fftconv_inverse_transform": (ip, [vp, ip, vp, vp, vp, ip]),
        "fftconv_profile_enable": (ip, [vp, ctypes.c_uint]),
        "fftconv_profile_read": (ip, [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_long)]),
        "fftconv_strerror": (ctypes.c_char_p, [ip]),
        "fftconv_paper_ram_bytes": (sz, [ip, ip, ip, ip]),
        "fftconv_contraction_flops": (ctypes.c_double, [vp]),
        "fftconv_tiling": (ip, [vp, ctypes.POINTER(ip * 2), ctypes.POINTER(ip * 2), ctypes.POINTER(ip * 2)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()


def strerror(status: int) -> str:
    return _lib.fftconv_strerror(int(status)).decode()


def paper_ram_bytes(S: int, n: int, f: int, fo: int) -> int:
    return int(_lib.fftconv_paper_ram_bytes(S, n, f, fo))


def _check(status: int, where: str):
    if status != FFTCONV_OK:
        raise FftconvError(status, where)


def _ptr(t, what: str):
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise ValueError(f"{what} must be a contiguous fp32 device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Plan:
    """One layer's plan plus (optionally) a torch-owned workspace.

    The passes are the C entry points of the same names; tensors must be
    contiguous fp32 device tensors of the shapes in include/fftconv.h.
    """

    def __init__(self, S: int, f: int, fo: int, n, k, flags: int = 0):
        """n, k: ints (square maps / kernels, the paper's notation) or (height, width) pairs."""
        self._h = ctypes.c_void_p()
        if isinstance(n, (tuple, list)) or isinstance(k, (tuple, list)):
            nh, nw = n if isinstance(n, (tuple, list)) else (n, n)
            kh, kw = k if isinstance(k, (tuple, list)) else (k, k)
            d = Desc2d(S, f, fo, nh, nw, kh, kw, flags)
            _check(_lib.fftconv_plan2d(ctypes.byref(self._h), ctypes.byref(d)), "fftconv_plan2d")
        else:
            nh = nw = n
            kh = kw = k
            d = Desc(S, f, fo, n, k, flags)
            _check(_lib.fftconv_plan(ctypes.byref(self._h), ctypes.byref(d)), "fftconv_plan")
        self.S, self.f, self.fo, self.n, self.k = S, f, fo, n, k
        self.nh, self.nw, self.kh, self.kw = nh, nw, kh, kw
        self.noh, self.now = nh - kh + 1, nw - kw + 1
        self.no = self.noh
        self.ws = None

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value and _lib is not None:
            _lib.fftconv_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    # -- queries ---------------------------------------------------------
    @property
    def fft_size(self) -> int:
        return int(_lib.fftconv_fft_size(self._h))

    @property
    def num_bins(self) -> int:
        return int(_lib.fftconv_num_bins(self._h))

    @property
    def workspace_bytes(self) -> int:
        return int(_lib.fftconv_workspace_bytes(self._h))

    @property
    def contraction_flops(self) -> float:
        return float(_lib.fftconv_contraction_flops(self._h))

    @property
    def tiling(self):
        """((Ly, Lx), tiles of y per axis, tiles of dx per axis); (0, 0) first if the layer is not tiled."""
        a, b, c = (ctypes.c_int * 2)(), (ctypes.c_int * 2)(), (ctypes.c_int * 2)()
        _check(_lib.fftconv_tiling(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fftconv_tiling")
        return tuple(a), tuple(b), tuple(c)

    def slot_offset(self, slot: int) -> int:
        return int(_lib.fftconv_slot_offset(self._h, slot))

    def slot_maps(self, slot: int) -> int:
        return int(_lib.fftconv_slot_maps(self._h, slot))

    def valid_slots(self) -> int:
        return int(_lib.fftconv_valid_slots(self._h))

    def invalidate(self, slots: int = SPEC_X | SPEC_W | SPEC_G):
        _check(_lib.fftconv_invalidate(self._h, slots), "fftconv_invalidate")

    # -- workspace (device memory is torch's; the library never allocates) --
    def alloc_workspace(self, device="cuda:0"):
        self.ws = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=device)
        return self.ws

    def _ws_ptr(self):
        if self.ws is None:
            self.alloc_workspace()
        p = self.ws.data_ptr()
        return ctypes.c_void_p((p + 255) // 256 * 256)

    def slot_view(self, slot: int):
        """The slot's spectrum as a [B, M, 2] fp32 view of the workspace."""
        B, M = self.num_bins, self.slot_maps(slot)
        if M < 0:
            raise ValueError(f"slot {slot} has no place of its own in this plan's workspace")
        base = self._ws_ptr().value - self.ws.data_ptr() + self.slot_offset(slot)
        return self.ws[base:base + 8 * B * M].view(torch.float32).view(B, M, 2)

    # -- passes ------------------------------------------------------------
    def fprop(self, x, w, y=None):
        if y is None:
            y = torch.empty((self.S, self.fo, self.noh, self.now), dtype=torch.float32, device=x.device)
        _check(_lib.fftconv_fprop(self._h, _ptr(x, "x"), _ptr(w, "w"), _ptr(y, "y"), self._ws_ptr(), _stream()),
               "fftconv_fprop")
        return y

    def bprop(self, g, w, dx=None):
        if dx is None:
            dx = torch.empty((self.S, self.f, self.nh, self.nw), dtype=torch.float32, device=g.device)
        _check(_lib.fftconv_bprop(self._h, _ptr(g, "g"), _ptr(w, "w"), _ptr(dx, "dx"), self._ws_ptr(), _stream()),
               "fftconv_bprop")
        return dx

    def accgrad(self, g, x, dw=None, accumulate: bool = False):
        if dw is None:
            if accumulate:
                raise ValueError("accumulate needs an existing dw")
            dw = torch.empty((self.fo, self.f, self.kh, self.kw), dtype=torch.float32, device=g.device)
        _check(_lib.fftconv_accgrad(self._h, _ptr(g, "g"), _ptr(x, "x"), _ptr(dw, "dw"), self._ws_ptr(), _stream(),
                                    1 if accumulate else 0), "fftconv_accgrad")
        return dw

    def pass_static(self, pass_id: int, a, b, out, accumulate: bool = False):
        """fftconv_pass_static: the pass on the library's own static scratch; allocates nothing
        (``out`` must exist)."""
        _check(_lib.fftconv_pass_static(self._h, pass_id, _ptr(a, "a"), _ptr(b, "b"), _ptr(out, "out"), _stream(),
                                        1 if accumulate else 0), "fftconv_pass_static")
        return out

    # -- single stages -----------------------------------------------------
    def forward_transform(self, slot: int, src):
        _check(_lib.fftconv_forward_transform(self._h, slot, _ptr(src, "src"), self._ws_ptr(), _stream()),
               "fftconv_forward_transform")

    def contract(self, pass_id: int):
        _check(_lib.fftconv_contract(self._h, pass_id, self._ws_ptr(), _stream()), "fftconv_contract")

    def inverse_transform(self, pass_id: int, dst, accumulate: bool = False):
        _check(_lib.fftconv_inverse_transform(self._h, pass_id, _ptr(dst, "dst"), self._ws_ptr(), _stream(),
                                              1 if accumulate else 0), "fftconv_inverse_transform")

    # -- stage timing --------------------------------------------------------
    def profile_enable(self, stages=True):
        """stages: True (all), False (none) or an iterable of stage names to bracket with events."""
        if stages is True:
            mask = PROFILE_ALL
        elif not stages:
            mask = 0
        else:
            mask = sum(1 << STAGE_NAMES.index(s) for s in stages)
        _check(_lib.fftconv_profile_enable(self._h, mask), "fftconv_profile_enable")

    def profile_read(self):
        """Returns {stage name: (total ms, launches)} since the last read."""
        ms = (ctypes.c_double * NUM_STAGES)()
        cnt = (ctypes.c_long * NUM_STAGES)()
        _check(_lib.fftconv_profile_read(self._h, ms, cnt), "fftconv_profile_read")
        return {STAGE_NAMES[i]: (float(ms[i]), int(cnt[i])) for i in range(NUM_STAGES)}
