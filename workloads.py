"""Seeded synthetic inputs for the PV-Tuning V-step re-encoding path.

This module only draws random tensors of the shapes and distributions of the
benchmark configurations; it holds none of the method's arithmetic (no target
formation, no scoring, no search, no dequantisation).  Both the CPU oracle's
tests and the HIP path's tests/bench read their inputs from here, so the two
sides see identical bytes.

The tensors stand in for real LLM weights / gradients: shapes follow the
Llama-2-7B linear layers (4096, 11008) and the 14336-wide MLP of the
Llama-3-8B / Mistral-7B class; quantiser shapes follow the paper's App. K
(one 16-bit codebook over groups of 8 or 16; two 8-bit codebooks over groups
of 8 with beam size 8).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Layout:
    out_features: int
    in_features: int
    group_size: int
    num_codebooks: int
    nbits: int

    @property
    def groups_per_row(self) -> int:
        return self.in_features // self.group_size

    @property
    def num_groups(self) -> int:
        return self.out_features * self.groups_per_row

    @property
    def codebook_size(self) -> int:
        return 1 << self.nbits


@dataclass
class Workload:
    name: str
    layout: Layout
    alpha: float
    tau: float
    beam_width: int
    W: np.ndarray          # f32 [out, in]
    G: np.ndarray          # f32 [out, in]
    codebooks: np.ndarray  # f32 [M, 2^B, g]
    scales: np.ndarray     # f32 [out]
    codes: np.ndarray      # u16 [out, in/g, M]
    meta: dict = field(default_factory=dict)

    @property
    def k(self) -> int:
        return num_selected(self.layout.num_groups, self.tau)


def num_selected(num_groups: int, tau: float) -> int:
    """Number of groups a fraction tau selects: floor(tau*N), but at least one."""
    return max(1, min(num_groups, int(np.floor(tau * num_groups + 1e-9))))


# name -> (out, in, g, M, B, sigma_w, sigma_g, alpha, scales, tau, beam)
_CONFIGS = {
    # small case the oracle finishes instantly
    "c1_256x256_1x8": (256, 256, 8, 1, 8, 0.02, 1e-3, 1.0, "ones", 1.0, 1),
    # Llama-2-7B q_proj, one 16-bit codebook, group 8 (the benchmark workload)
    "c2_4096x4096_1x16": (4096, 4096, 8, 1, 16, 0.02, 1e-4, 1.0, "uniform", 0.01, 1),
    # Llama-2-7B MLP up/gate, two 8-bit codebooks, beam 8
    "c3_11008x4096_2x8": (11008, 4096, 8, 2, 8, 0.02, 1e-4, 1.0, "uniform", 0.05, 8),
    # 1-bit configs: group 16, one 16-bit codebook
    "c5a_14336x4096_1x16g16": (14336, 4096, 16, 1, 16, 0.02, 1e-4, 1.0, "uniform", 0.05, 1),
    "c5b_4096x14336_1x16g16": (4096, 14336, 16, 1, 16, 0.02, 1e-4, 1.0, "uniform", 0.05, 1),
}

# The 7 linear layers of one Llama-2-7B decoder block (the full-stack config
# repeats this block 32 times with fresh seeds): name -> (out, in)
LLAMA2_7B_BLOCK = {
    "q_proj": (4096, 4096), "k_proj": (4096, 4096), "v_proj": (4096, 4096),
    "o_proj": (4096, 4096), "gate_proj": (11008, 4096), "up_proj": (11008, 4096),
    "down_proj": (4096, 11008),
}


def config_names():
    return list(_CONFIGS)


def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, tensor_id]))


def make(out_features: int, in_features: int, group_size: int, num_codebooks: int,
         nbits: int, *, sigma_w: float = 0.02, sigma_g: float = 1e-4,
         sigma_c: float = 0.02, alpha: float = 1.0, scales: str = "uniform",
         tau: float = 0.01, beam_width: int = 1, seed: int = 0,
         name: str = "custom", structured: bool = False) -> Workload:
    """Draw one weight matrix' worth of inputs.

    structured=False: W is a dense Gaussian matrix as the configs state, the
    initial codes are uniform random.  structured=True: the caller is expected
    to overwrite W with the dequantised initial codes (done by whoever owns a
    dequantiser; this module has none).
    """
    lay = Layout(out_features, in_features, group_size, num_codebooks, nbits)
    assert in_features % group_size == 0
    W = _rng(seed, 1).standard_normal((out_features, in_features), dtype=np.float32)
    W *= np.float32(sigma_w)
    G = _rng(seed, 2).standard_normal((out_features, in_features), dtype=np.float32)
    G *= np.float32(sigma_g)
    cb = _rng(seed, 3).standard_normal((num_codebooks, lay.codebook_size, group_size),
                                       dtype=np.float32)
    cb *= np.float32(sigma_c)
    if scales == "ones":
        sc = np.ones(out_features, dtype=np.float32)
    elif scales == "uniform":
        sc = (_rng(seed, 4).random(out_features, dtype=np.float32) + np.float32(0.5))
    else:
        raise ValueError(scales)
    codes = _rng(seed, 5).integers(0, lay.codebook_size,
                                   size=(out_features, lay.groups_per_row, num_codebooks),
                                   dtype=np.uint16 if nbits < 16 else np.uint32)
    codes = codes.astype(np.uint16)
    return Workload(name=name, layout=lay, alpha=float(alpha), tau=float(tau),
                    beam_width=int(beam_width), W=W, G=G, codebooks=cb,
                    scales=sc.astype(np.float32), codes=codes,
                    meta={"seed": seed, "structured": structured})


def make_config(name: str, seed: int = 0, *, out_features: int | None = None,
                in_features: int | None = None, tau: float | None = None) -> Workload:
    """One of the named benchmark configurations, optionally shrunk in shape."""
    (o, i, g, M, B, sw, sg, a, sc, t, beam) = _CONFIGS[name]
    o = out_features or o
    i = in_features or i
    t = t if tau is None else tau
    return make(o, i, g, M, B, sigma_w=sw, sigma_g=sg, alpha=a, scales=sc, tau=t,
                beam_width=beam, seed=seed, name=name)


def make_block_matrix(layer: int, proj: str, seed: int = 0) -> Workload:
    """One matrix of the Llama-2-7B-shaped stack (1x16 codebook, group 8, tau 0.01)."""
    o, i = LLAMA2_7B_BLOCK[proj]
    pid = list(LLAMA2_7B_BLOCK).index(proj)
    return make(o, i, 8, 1, 16, sigma_g=1e-4, tau=0.01,
                seed=(seed * 1_000_003 + layer * 16 + pid + 1),
                name=f"c4_layer{layer}_{proj}")


def make_scalar(out_features: int, in_features: int, block: int, nbits: int, *, sigma_w: float = 0.02,
                sigma_g: float = 1e-3, seed: int = 0):
    """Inputs for the scalar uniform-grid representation of App. K (block-wise scale and zero
    point along the input dimension): (W, G, codes u8 [out, in], scales, zeros [out, in/block])."""
    assert in_features % block == 0
    W = _rng(seed, 11).standard_normal((out_features, in_features), dtype=np.float32) * np.float32(sigma_w)
    G = _rng(seed, 12).standard_normal((out_features, in_features), dtype=np.float32) * np.float32(sigma_g)
    codes = _rng(seed, 13).integers(0, 1 << nbits, size=(out_features, in_features), dtype=np.uint8)
    shape = (out_features, in_features // block)
    # a grid that covers about +-3 sigma of the weights
    scales = (_rng(seed, 14).random(shape, dtype=np.float32) + np.float32(0.5)) \
        * np.float32(6.0 * sigma_w / ((1 << nbits) - 1))
    zeros = np.float32(((1 << nbits) - 1) / 2.0) + (_rng(seed, 15).random(shape, dtype=np.float32)
                                                    - np.float32(0.5))
    return W.astype(np.float32), G.astype(np.float32), codes, scales.astype(np.float32), zeros.astype(np.float32)
