"""ctypes binding of libpv.so: same names as the C ABI, no arithmetic here.

Tensors are torch CUDA tensors (PyTorch is used for device memory and streams
only).  The library must have been built (see __graft_entry__.build); a missing
library is an error, there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
_LIB_PATH = _PKG / "libpv.so"
_lib = None

KERNEL_IDS = {
    "encode_targets": 0, "group_scores": 1, "select": 2, "prep": 3, "score_mfma": 4,
    "rerank": 5, "exact_scan": 6, "beam": 7, "dequantize": 8, "trust_ratio": 9, "pstep": 10, "stochastic": 13,
    "probe_copy": 11, "probe_mfma": 12,
}


class PVError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"pv status {status}: {text}")
        self.status = status


class _CLayout(ctypes.Structure):
    _fields_ = [("out_features", ctypes.c_int64), ("in_features", ctypes.c_int64),
                ("group_size", ctypes.c_int32), ("num_codebooks", ctypes.c_int32),
                ("nbits", ctypes.c_int32)]


@dataclass(frozen=True)
class Layout:
    out_features: int
    in_features: int
    group_size: int
    num_codebooks: int
    nbits: int

    def c(self) -> _CLayout:
        return _CLayout(self.out_features, self.in_features, self.group_size,
                        self.num_codebooks, self.nbits)

    @property
    def num_groups(self) -> int:
        return self.out_features * (self.in_features // self.group_size)


def library_path() -> Path:
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(str(_LIB_PATH))
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    lp = ctypes.POINTER(_CLayout)
    lib.pv_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp]
    lib.pv_destroy.argtypes = [vp]
    lib.pv_destroy.restype = None
    lib.pv_last_error.argtypes = [vp]
    lib.pv_last_error.restype = ctypes.c_char_p
    lib.pv_encode_targets.argtypes = [vp, lp, vp, vp, f32, vp]
    lib.pv_encode_targets_adam.argtypes = [vp, lp, vp, vp, vp, vp, i64, f32, f32, f32, f32, vp]
    lib.pv_select_topk_groups.argtypes = [vp, lp, vp, vp, i64, vp, vp]
    lib.pv_select_topk_groups_noalloc.argtypes = [vp, lp, vp, vp, i64, vp, vp]
    lib.pv_encode_targets_adam_select.argtypes = [vp, lp, vp, vp, vp, vp, i64, f32, f32, f32, f32, vp,
                                                  i64, vp, vp]
    lib.pv_encode_targets_select.argtypes = [vp, lp, vp, vp, f32, vp, i64, vp, vp]
    lib.pv_reencode_groups.argtypes = [vp, lp, vp, vp, vp, vp, i64, i32, vp, vp]
    lib.pv_reencode_groups_stochastic.argtypes = [vp, lp, vp, vp, vp, vp, i64, i32, ctypes.c_uint64, vp, vp]
    lib.pv_dequantize.argtypes = [vp, lp, vp, vp, vp, vp]
    lib.pv_dequantize_groups.argtypes = [vp, lp, vp, vp, vp, vp, i64, vp]
    lib.pv_codebook_grads.argtypes = [vp, lp, vp, vp, vp, vp, vp, vp]
    lib.pv_dequantize_scalar.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.pv_reencode_scalar.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, i64, vp, vp]
    lib.pv_reencode_trust_ratio.argtypes = [vp, lp, vp, vp, vp, vp, i64, i64, ctypes.c_double, i32,
                                            vp, vp, vp, vp]
    lib.pv_set_search_mode.argtypes = [vp, ctypes.c_int]
    lib.pv_timing_enable.argtypes = [vp, ctypes.c_int]
    lib.pv_timing_reset.argtypes = [vp]
    lib.pv_timing_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                   ctypes.POINTER(i64)]
    lib.pv_reencode_stats.argtypes = [vp, ctypes.POINTER(i64)]
    lib.pv_probe_copy.argtypes = [vp, vp, vp, i64]
    lib.pv_probe_mfma_f16.argtypes = [vp, i64, vp, ctypes.POINTER(i64)]
    for name in ("pv_create", "pv_select_topk_groups_noalloc", "pv_encode_targets", "pv_encode_targets_adam", "pv_select_topk_groups",
                 "pv_encode_targets_adam_select",
                 "pv_encode_targets_select", "pv_reencode_groups", "pv_reencode_groups_stochastic",
                 "pv_reencode_trust_ratio",
                 "pv_codebook_grads", "pv_dequantize_scalar", "pv_reencode_scalar",
                 "pv_dequantize_groups",
                 "pv_dequantize", "pv_set_search_mode", "pv_timing_enable", "pv_timing_reset",
                 "pv_timing_read", "pv_reencode_stats", "pv_probe_copy", "pv_probe_mfma_f16"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _dev_ptr(t, dtype, what: str, allow_none: bool = False):
    if t is None:
        if allow_none:
            return None
        raise TypeError(f"{what} is None")
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a CUDA tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError(f"{what} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


class PVContext:
    """One library context bound to a device and a stream (default: torch's current stream)."""

    def __init__(self, device: int = 0, stream: "torch.cuda.Stream | None" = None):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.device = device
        with torch.cuda.device(device):
            s = stream if stream is not None else torch.cuda.current_stream(device)
        self.stream = s
        st = self._lib.pv_create(ctypes.byref(self._h), device, ctypes.c_void_p(s.cuda_stream))
        if st != 0:
            raise PVError(st, "pv_create failed")

    def close(self):
        if self._h:
            self._lib.pv_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != 0:
            raise PVError(st, self._lib.pv_last_error(self._h).decode())

    # ---- the four calls of the path -------------------------------------
    def pv_encode_targets(self, layout: Layout, W, G, alpha: float, T):
        lay = layout.c()
        self._check(self._lib.pv_encode_targets(
            self._h, ctypes.byref(lay), _dev_ptr(W, torch.float32, "W"),
            _dev_ptr(G, torch.float32, "G"), float(alpha), _dev_ptr(T, torch.float32, "T")))

    def pv_encode_targets_adam(self, layout: Layout, W, G, m, v, step: int, lr: float,
                               beta1: float, beta2: float, eps: float, T):
        lay = layout.c()
        self._check(self._lib.pv_encode_targets_adam(
            self._h, ctypes.byref(lay), _dev_ptr(W, torch.float32, "W"),
            _dev_ptr(G, torch.float32, "G"), _dev_ptr(m, torch.float32, "m"),
            _dev_ptr(v, torch.float32, "v"), int(step), float(lr), float(beta1), float(beta2),
            float(eps), _dev_ptr(T, torch.float32, "T")))

    def pv_encode_targets_adam_select(self, layout: Layout, W, G, m, v, step: int, lr: float,
                                      beta1: float, beta2: float, eps: float, T, k: int, out_idx,
                                      group_scores=None):
        lay = layout.c()
        self._check(self._lib.pv_encode_targets_adam_select(
            self._h, ctypes.byref(lay), _dev_ptr(W, torch.float32, "W"),
            _dev_ptr(G, torch.float32, "G"), _dev_ptr(m, torch.float32, "m"),
            _dev_ptr(v, torch.float32, "v"), int(step), float(lr), float(beta1), float(beta2),
            float(eps), _dev_ptr(T, torch.float32, "T"), int(k),
            _dev_ptr(out_idx, torch.int32, "out_idx", allow_none=(k == 0)),
            _dev_ptr(group_scores, torch.float32, "group_scores", allow_none=True)))

    def pv_select_topk_groups(self, layout: Layout, T, W, k: int, out_idx, group_scores=None):
        lay = layout.c()
        self._check(self._lib.pv_select_topk_groups(
            self._h, ctypes.byref(lay), _dev_ptr(T, torch.float32, "T"),
            _dev_ptr(W, torch.float32, "W"), int(k),
            _dev_ptr(out_idx, torch.int32, "out_idx", allow_none=(k == 0)),
            _dev_ptr(group_scores, torch.float32, "group_scores", allow_none=True)))

    def pv_select_topk_groups_noalloc(self, layout: Layout, T, W, k: int, out_idx, group_scores=None):
        lay = layout.c()
        self._check(self._lib.pv_select_topk_groups_noalloc(
            self._h, ctypes.byref(lay), _dev_ptr(T, torch.float32, "T"),
            _dev_ptr(W, torch.float32, "W"), int(k),
            _dev_ptr(out_idx, torch.int32, "out_idx", allow_none=(k == 0)),
            _dev_ptr(group_scores, torch.float32, "group_scores", allow_none=True)))

    def pv_encode_targets_select(self, layout: Layout, W, G, alpha: float, T, k: int, out_idx,
                                 group_scores=None):
        lay = layout.c()
        self._check(self._lib.pv_encode_targets_select(
            self._h, ctypes.byref(lay), _dev_ptr(W, torch.float32, "W"),
            _dev_ptr(G, torch.float32, "G"), float(alpha), _dev_ptr(T, torch.float32, "T"), int(k),
            _dev_ptr(out_idx, torch.int32, "out_idx", allow_none=(k == 0)),
            _dev_ptr(group_scores, torch.float32, "group_scores", allow_none=True)))

    def pv_reencode_groups(self, layout: Layout, T, codebooks, scales, group_idx, k: int,
                           beam_width: int, codes, num_changed=None):
        lay = layout.c()
        self._check(self._lib.pv_reencode_groups(
            self._h, ctypes.byref(lay), _dev_ptr(T, torch.float32, "T"),
            _dev_ptr(codebooks, torch.float32, "codebooks"),
            _dev_ptr(scales, torch.float32, "scales"),
            _dev_ptr(group_idx, torch.int32, "group_idx", allow_none=(k == 0)), int(k),
            int(beam_width), _dev_ptr(codes, torch.uint16, "codes"),
            _dev_ptr(num_changed, torch.int64, "num_changed", allow_none=True)))

    def pv_reencode_groups_stochastic(self, layout: Layout, T, codebooks, scales, group_idx, k: int,
                                      power: int, seed: int, codes, num_changed=None):
        lay = layout.c()
        self._check(self._lib.pv_reencode_groups_stochastic(
            self._h, ctypes.byref(lay), _dev_ptr(T, torch.float32, "T"),
            _dev_ptr(codebooks, torch.float32, "codebooks"),
            _dev_ptr(scales, torch.float32, "scales"),
            _dev_ptr(group_idx, torch.int32, "group_idx", allow_none=(k == 0)), int(k),
            int(power), int(seed) & (2 ** 64 - 1), _dev_ptr(codes, torch.uint16, "codes"),
            _dev_ptr(num_changed, torch.int64, "num_changed", allow_none=True)))

    def pv_reencode_trust_ratio(self, layout: Layout, T, W, codebooks, scales, k_max: int,
                                chunk: int, ratio: float, beam_width: int, codes, rank_idx,
                                num_applied, stats=None):
        lay = layout.c()
        self._check(self._lib.pv_reencode_trust_ratio(
            self._h, ctypes.byref(lay), _dev_ptr(T, torch.float32, "T"),
            _dev_ptr(W, torch.float32, "W"), _dev_ptr(codebooks, torch.float32, "codebooks"),
            _dev_ptr(scales, torch.float32, "scales"), int(k_max), int(chunk), float(ratio),
            int(beam_width), _dev_ptr(codes, torch.uint16, "codes"),
            _dev_ptr(rank_idx, torch.int32, "rank_idx", allow_none=True),
            _dev_ptr(num_applied, torch.int64, "num_applied"),
            _dev_ptr(stats, torch.float64, "stats", allow_none=True)))

    def pv_dequantize_groups(self, layout: Layout, codes, codebooks, scales, group_idx, k: int, W_out):
        lay = layout.c()
        self._check(self._lib.pv_dequantize_groups(
            self._h, ctypes.byref(lay), _dev_ptr(codes, torch.uint16, "codes"),
            _dev_ptr(codebooks, torch.float32, "codebooks"), _dev_ptr(scales, torch.float32, "scales"),
            _dev_ptr(group_idx, torch.int32, "group_idx", allow_none=(k == 0)), int(k),
            _dev_ptr(W_out, torch.float32, "W_out")))

    def pv_codebook_grads(self, layout: Layout, G, codes, codebooks, scales, grad_codebooks,
                          grad_scales=None):
        lay = layout.c()
        self._check(self._lib.pv_codebook_grads(
            self._h, ctypes.byref(lay), _dev_ptr(G, torch.float32, "G"),
            _dev_ptr(codes, torch.uint16, "codes"), _dev_ptr(codebooks, torch.float32, "codebooks"),
            _dev_ptr(scales, torch.float32, "scales"),
            _dev_ptr(grad_codebooks, torch.float32, "grad_codebooks"),
            _dev_ptr(grad_scales, torch.float32, "grad_scales", allow_none=True)))

    def pv_dequantize_scalar(self, out_features: int, in_features: int, block_size: int, nbits: int,
                             codes, scales, zeros, W_out):
        self._check(self._lib.pv_dequantize_scalar(
            self._h, int(out_features), int(in_features), int(block_size), int(nbits),
            _dev_ptr(codes, torch.uint8, "codes"), _dev_ptr(scales, torch.float32, "scales"),
            _dev_ptr(zeros, torch.float32, "zeros"), _dev_ptr(W_out, torch.float32, "W_out")))

    def pv_reencode_scalar(self, out_features: int, in_features: int, block_size: int, nbits: int,
                           T, scales, zeros, weight_idx, k: int, codes, num_changed=None):
        self._check(self._lib.pv_reencode_scalar(
            self._h, int(out_features), int(in_features), int(block_size), int(nbits),
            _dev_ptr(T, torch.float32, "T"), _dev_ptr(scales, torch.float32, "scales"),
            _dev_ptr(zeros, torch.float32, "zeros"),
            _dev_ptr(weight_idx, torch.int32, "weight_idx", allow_none=(k == 0)), int(k),
            _dev_ptr(codes, torch.uint8, "codes"),
            _dev_ptr(num_changed, torch.int64, "num_changed", allow_none=True)))

    def pv_dequantize(self, layout: Layout, codes, codebooks, scales, W_out):
        lay = layout.c()
        self._check(self._lib.pv_dequantize(
            self._h, ctypes.byref(lay), _dev_ptr(codes, torch.uint16, "codes"),
            _dev_ptr(codebooks, torch.float32, "codebooks"),
            _dev_ptr(scales, torch.float32, "scales"), _dev_ptr(W_out, torch.float32, "W_out")))

    # ---- instrumentation --------------------------------------------------
    def pv_set_search_mode(self, mode: int):
        self._check(self._lib.pv_set_search_mode(self._h, int(mode)))

    def pv_timing_enable(self, on: bool):
        self._check(self._lib.pv_timing_enable(self._h, int(bool(on))))

    def pv_timing_reset(self):
        self._check(self._lib.pv_timing_reset(self._h))

    def pv_timing_read(self, kernel: "int | str"):
        kid = KERNEL_IDS[kernel] if isinstance(kernel, str) else int(kernel)
        ms, n = ctypes.c_double(0), ctypes.c_int64(0)
        self._check(self._lib.pv_timing_read(self._h, kid, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def pv_probe_copy(self, dst, src):
        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != nbytes:
            raise ValueError("dst and src differ in size")
        self._check(self._lib.pv_probe_copy(self._h, ctypes.c_void_p(dst.data_ptr()),
                                            ctypes.c_void_p(src.data_ptr()), int(nbytes)))

    def pv_probe_mfma_f16(self, iters: int, sink):
        waves = ctypes.c_int64(0)
        self._check(self._lib.pv_probe_mfma_f16(self._h, int(iters), _dev_ptr(sink, torch.float32, "sink"),
                                                ctypes.byref(waves)))
        return waves.value

    def pv_reencode_stats(self):
        arr = (ctypes.c_int64 * 4)()
        self._check(self._lib.pv_reencode_stats(self._h, arr))
        return {"filtered": arr[0], "fallback": arr[1], "reranked_candidates": arr[2],
                "exact": arr[3]}
