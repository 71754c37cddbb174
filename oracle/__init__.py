"""ctypes front end of the CPU oracle (oracle/pvo.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "pvo.c"
# PVO_SANITIZE=1: a second build with the address and undefined-behaviour sanitizers of gcc, for
# running the CPU tests once under them:
#   PVO_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
#       python -m pytest tests -m "not gpu"
_SANITIZE = os.environ.get("PVO_SANITIZE", "0") not in ("", "0")
_LIB = _HERE / ("libpvo_san.so" if _SANITIZE else "libpvo.so")

_lib = None


def build(force: bool = False) -> Path:
    """Compile pvo.c with gcc (no contraction, OpenMP over groups)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        if _SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=undefined"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i64, i32, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_float
        p = ctypes.c_void_p
        lib.pvo_encode_targets.argtypes = [i64, i64, p, p, f32, p]
        lib.pvo_select_topk_groups.argtypes = [i64, i64, i32, p, p, i64, p, p]
        lib.pvo_reencode_groups.argtypes = [i64, i64, i32, i32, i32, p, p, p, p, i64, i32, i32,
                                            p, p, p, p, p]
        lib.pvo_reencode_stochastic.argtypes = [i64, i64, i32, i32, p, p, p, p, i64, i32, ctypes.c_uint64,
                                                p, p, p, p, p, p, p]
        lib.pvo_random_bits.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.pvo_random_bits.restype = ctypes.c_uint64
        lib.pvo_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.pvo_uniform.restype = ctypes.c_double
        lib.pvo_group_objective.argtypes = [i64, i64, i32, i32, i32, p, p, p, p, i64, p, p]
        lib.pvo_dequantize.argtypes = [i64, i64, i32, i32, i32, p, p, p, p]
        lib.pvo_encode_targets_adam.argtypes = [i64, i64, p, p, p, p, i64, f32, f32, f32, f32, p]
        lib.pvo_encode_targets_adam.restype = ctypes.c_int
        lib.pvo_codebook_grads.argtypes = [i64, i64, i32, i32, i32, p, p, p, p, p, p]
        lib.pvo_codebook_grads.restype = ctypes.c_int
        lib.pvo_dequantize_scalar.argtypes = [i64, i64, i32, i32, p, p, p, p]
        lib.pvo_reencode_scalar.argtypes = [i64, i64, i32, i32, p, p, p, p, i64, p, p]
        lib.pvo_dequantize_scalar.restype = lib.pvo_reencode_scalar.restype = ctypes.c_int
        f64 = ctypes.c_double
        lib.pvo_reencode_trust_ratio.argtypes = [i64, i64, i32, i32, i32, p, p, p, p, i64, i64, f64,
                                                 i32, p, p, p, p]
        lib.pvo_reencode_trust_ratio.restype = ctypes.c_int
        for f in (lib.pvo_encode_targets, lib.pvo_select_topk_groups, lib.pvo_reencode_groups,
                  lib.pvo_group_objective, lib.pvo_dequantize, lib.pvo_num_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def num_threads() -> int:
    return int(_load().pvo_num_threads())


def encode_targets(W, G, alpha: float) -> np.ndarray:
    W, G = _f32(W), _f32(G)
    assert W.shape == G.shape and W.ndim == 2
    T = np.empty_like(W)
    rc = _load().pvo_encode_targets(W.shape[0], W.shape[1], _ptr(W), _ptr(G), float(alpha), _ptr(T))
    if rc:
        raise ValueError("pvo_encode_targets failed")
    return T


def encode_targets_adam(W, G, m, v, t: int, lr: float, beta1: float = 0.9, beta2: float = 0.95,
                        eps: float = 1e-8):
    """Returns (T, m_new, v_new); the inputs are left untouched."""
    W, G = _f32(W), _f32(G)
    m2, v2 = _f32(m).copy(), _f32(v).copy()
    assert W.shape == G.shape == m2.shape == v2.shape and W.ndim == 2
    T = np.empty_like(W)
    rc = _load().pvo_encode_targets_adam(W.shape[0], W.shape[1], _ptr(W), _ptr(G), _ptr(m2), _ptr(v2),
                                         int(t), float(lr), float(beta1), float(beta2), float(eps),
                                         _ptr(T))
    if rc:
        raise ValueError("pvo_encode_targets_adam failed")
    return T, m2, v2


def select_topk_groups(T, W, group_size: int, k: int, return_scores: bool = False):
    T, W = _f32(T), _f32(W)
    out_f, in_f = T.shape
    N = out_f * (in_f // group_size)
    idx = np.empty(max(k, 0), dtype=np.int32)
    scores = np.empty(N, dtype=np.float32) if return_scores else None
    rc = _load().pvo_select_topk_groups(out_f, in_f, group_size, _ptr(T), _ptr(W), k, _ptr(idx),
                                        _ptr(scores))
    if rc:
        raise ValueError("pvo_select_topk_groups failed")
    return (idx, scores) if return_scores else idx


def reencode_groups(T, codebooks, scales, group_idx, codes, beam_width: int = 1,
                    use_beam: bool = False):
    """Returns (new_codes, info) and leaves `codes` untouched."""
    T = _f32(T)
    cb = _f32(codebooks)
    sc = _f32(scales)
    M, csize, g = cb.shape
    B = int(csize).bit_length() - 1
    assert (1 << B) == csize
    out_f, in_f = T.shape
    idx = np.ascontiguousarray(group_idx, dtype=np.int32)
    k = idx.shape[0]
    new = np.ascontiguousarray(codes, dtype=np.uint16).copy()
    assert new.shape == (out_f, in_f // g, M), new.shape
    changed = ctypes.c_int64(0)
    near = np.zeros(k, dtype=np.uint8)
    obj_new = np.zeros(k, dtype=np.float64)
    obj_prev = np.zeros(k, dtype=np.float64)
    rc = _load().pvo_reencode_groups(out_f, in_f, g, M, B, _ptr(T), _ptr(cb), _ptr(sc), _ptr(idx),
                                     k, int(beam_width), int(bool(use_beam)), _ptr(new),
                                     ctypes.addressof(changed), _ptr(near), _ptr(obj_new),
                                     _ptr(obj_prev))
    if rc:
        raise ValueError("pvo_reencode_groups failed")
    return new, {"num_changed": int(changed.value), "near_tie": near.astype(bool),
                 "obj_new": obj_new, "obj_prev": obj_prev}


def uniform(seed: int, counter: int) -> float:
    """The variate in [0, 1) that the stochastic rounding draws for group `counter`."""
    return float(_load().pvo_uniform(int(seed) & (2 ** 64 - 1), int(counter)))


def random_bits(seed: int, counter: int) -> int:
    return int(_load().pvo_random_bits(int(seed) & (2 ** 64 - 1), int(counter)))


def reencode_stochastic(T, codebooks, scales, group_idx, codes, power: int = 5, seed: int = 0):
    """App. F, K = 2 nearest codewords, p proportional to distance^-power (App. K: power 5).
    Returns (new_codes, info) and leaves `codes` untouched."""
    T = _f32(T)
    cb = _f32(codebooks)
    sc = _f32(scales)
    M, csize, g = cb.shape
    if M != 1:
        raise ValueError("stochastic rounding is defined for one codebook")
    B = int(csize).bit_length() - 1
    assert (1 << B) == csize
    out_f, in_f = T.shape
    idx = np.ascontiguousarray(group_idx, dtype=np.int32)
    k = idx.shape[0]
    new = np.ascontiguousarray(codes, dtype=np.uint16).copy()
    assert new.shape == (out_f, in_f // g, 1), new.shape
    changed = ctypes.c_int64(0)
    two = np.zeros((k, 2), dtype=np.int32)
    obj = np.zeros((k, 2), dtype=np.float64)
    pn = np.zeros(k, dtype=np.float64)
    u = np.zeros(k, dtype=np.float64)
    near = np.zeros(k, dtype=np.uint8)
    rc = _load().pvo_reencode_stochastic(out_f, in_f, g, B, _ptr(T), _ptr(cb), _ptr(sc), _ptr(idx), k,
                                         int(power), int(seed) & (2 ** 64 - 1), _ptr(new),
                                         ctypes.addressof(changed), _ptr(two), _ptr(obj), _ptr(pn),
                                         _ptr(u), _ptr(near))
    if rc:
        raise ValueError("pvo_reencode_stochastic failed")
    return new, {"num_changed": changed.value, "nearest_two": two, "objective_two": obj,
                 "p_nearest": pn, "variate": u, "near_tie": near.astype(bool)}


def ste_step(buffer, G, alpha: float, codebooks, scales, codes, k=None, beam_width: int = 1):
    """One step of straight-through estimation (App. E): the auxiliary full-precision buffer takes
    the gradient step (computed at the quantised weights, passed in as G), then the codes are moved
    to approximate the buffer best in L2.  k = None re-encodes every group (plain STE); with k the
    step is restricted to the k groups whose buffer is farthest from the current quantised weights
    (the combination of subspace updates with STE, Sec. 4.3).  Returns (buffer, codes, info)."""
    cb = _f32(codebooks)
    g = cb.shape[2]
    new_buffer = encode_targets(buffer, G, alpha)
    out_f, in_f = new_buffer.shape
    if k is None:
        idx = np.arange(out_f * (in_f // g), dtype=np.int32)
    else:
        idx = select_topk_groups(new_buffer, dequantize(codes, codebooks, scales), g, k)
    new_codes, info = reencode_groups(new_buffer, codebooks, scales, idx, codes, beam_width=beam_width)
    info["group_idx"] = idx
    return new_buffer, new_codes, info


def reencode_trust_ratio(T, W, codebooks, scales, codes, k_max: int, chunk: int, ratio: float,
                         beam_width: int = 1):
    """Returns (new_codes, info); info: rank_idx [k_max] (selection order), num_applied,
    change_sq (squared change of the kept groups), norm_sq (||x^k||^2)."""
    T, W = _f32(T), _f32(W)
    cb = _f32(codebooks)
    sc = _f32(scales)
    M, csize, g = cb.shape
    B = int(csize).bit_length() - 1
    out_f, in_f = T.shape
    new = np.ascontiguousarray(codes, dtype=np.uint16).copy()
    assert new.shape == (out_f, in_f // g, M), new.shape
    rank = np.empty(max(k_max, 1), dtype=np.int32)
    applied = ctypes.c_int64(0)
    stats = np.zeros(2, dtype=np.float64)
    rc = _load().pvo_reencode_trust_ratio(out_f, in_f, g, M, B, _ptr(T), _ptr(W), _ptr(cb),
                                          _ptr(sc), int(k_max), int(chunk), float(ratio),
                                          int(beam_width), _ptr(new), _ptr(rank),
                                          ctypes.addressof(applied), _ptr(stats))
    if rc:
        raise ValueError("pvo_reencode_trust_ratio failed")
    return new, {"rank_idx": rank[:k_max], "num_applied": int(applied.value),
                 "change_sq": float(stats[0]), "norm_sq": float(stats[1])}


def dequantize_scalar(codes, scales, zeros, block: int, nbits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    sc, zp = _f32(scales), _f32(zeros)
    out_f, in_f = codes.shape
    assert sc.shape == zp.shape == (out_f, in_f // block)
    W = np.empty((out_f, in_f), dtype=np.float32)
    rc = _load().pvo_dequantize_scalar(out_f, in_f, int(block), int(nbits), _ptr(codes), _ptr(sc),
                                       _ptr(zp), _ptr(W))
    if rc:
        raise ValueError("pvo_dequantize_scalar failed")
    return W


def reencode_scalar(T, scales, zeros, weight_idx, codes, block: int, nbits: int):
    """Returns (new_codes, num_changed); `codes` is left untouched."""
    T = _f32(T)
    sc, zp = _f32(scales), _f32(zeros)
    out_f, in_f = T.shape
    idx = np.ascontiguousarray(weight_idx, dtype=np.int32)
    new = np.ascontiguousarray(codes, dtype=np.uint8).copy()
    assert new.shape == T.shape
    changed = ctypes.c_int64(0)
    rc = _load().pvo_reencode_scalar(out_f, in_f, int(block), int(nbits), _ptr(T), _ptr(sc), _ptr(zp),
                                     _ptr(idx), idx.shape[0], _ptr(new), ctypes.addressof(changed))
    if rc:
        raise ValueError("pvo_reencode_scalar failed")
    return new, int(changed.value)


def codebook_grads(G, codes, codebooks, scales):
    """Returns (grad_codebooks f32 [M, 2^B, g], grad_scales f32 [out])."""
    G = _f32(G)
    cb = _f32(codebooks)
    sc = _f32(scales)
    M, csize, g = cb.shape
    B = int(csize).bit_length() - 1
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    out_f, in_f = G.shape
    assert codes.shape == (out_f, in_f // g, M)
    gc = np.empty_like(cb)
    gs = np.empty(out_f, dtype=np.float32)
    rc = _load().pvo_codebook_grads(out_f, in_f, g, M, B, _ptr(G), _ptr(codes), _ptr(cb), _ptr(sc),
                                    _ptr(gc), _ptr(gs))
    if rc:
        raise ValueError("pvo_codebook_grads failed")
    return gc, gs


def group_objective(T, codebooks, scales, group_idx, tuples) -> np.ndarray:
    T = _f32(T)
    cb = _f32(codebooks)
    sc = _f32(scales)
    M, csize, g = cb.shape
    B = int(csize).bit_length() - 1
    out_f, in_f = T.shape
    idx = np.ascontiguousarray(group_idx, dtype=np.int32)
    tup = np.ascontiguousarray(tuples, dtype=np.uint16).reshape(idx.shape[0], M)
    obj = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().pvo_group_objective(out_f, in_f, g, M, B, _ptr(T), _ptr(cb), _ptr(sc), _ptr(idx),
                                     idx.shape[0], _ptr(tup), _ptr(obj))
    if rc:
        raise ValueError("pvo_group_objective failed")
    return obj


def dequantize(codes, codebooks, scales) -> np.ndarray:
    cb = _f32(codebooks)
    sc = _f32(scales)
    M, csize, g = cb.shape
    B = int(csize).bit_length() - 1
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    out_f, gpr, M2 = codes.shape
    assert M2 == M
    W = np.empty((out_f, gpr * g), dtype=np.float32)
    rc = _load().pvo_dequantize(out_f, gpr * g, g, M, B, _ptr(codes), _ptr(cb), _ptr(sc), _ptr(W))
    if rc:
        raise ValueError("pvo_dequantize failed")
    return W
