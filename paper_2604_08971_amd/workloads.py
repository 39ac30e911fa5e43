"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and lays out arrays: it contains none of
the method's arithmetic, so both the CPU oracle's tests and the GPU library's
tests may use it.  Everything is numpy on the host.

A workload stands in for "several sensor streams at different rates
concatenated into one token sequence, with random sensor dropout" (Sec. 4.2,
Sec. 4.4 of the paper); the paper's datasets are not reproduced.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np


def to_bf16_values(a: np.ndarray) -> np.ndarray:
    """Return fp32 array whose values are the nearest bf16 numbers (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_f16_values(a: np.ndarray) -> np.ndarray:
    """Return fp32 array whose values are the nearest IEEE binary16 numbers (ties to even)."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def storage_rounding(dtype: str):
    """The map that makes an fp32 array hold values of the model's storage type ("f32", "bf16" or "f16")."""
    if dtype == "bf16":
        return to_bf16_values
    if dtype == "f16":
        return to_f16_values
    return lambda a: np.ascontiguousarray(a, dtype=np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an fp32 array that already holds bf16 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def keep_count(ratio: float, n: int) -> int:
    """Keep ratio -> integer count, rounded half up, at least one unit."""
    return int(min(n, max(1, math.floor(ratio * n + 0.5))))


@dataclass
class Spec:
    """Shape of one workload (the five named ones are in CONFIGS)."""
    name: str
    dtype: str                      # "f32" | "bf16" | "f16" (the FP16 build of the library)
    B: int
    seg_tokens: Sequence[int]       # tokens per modality, in sequence order
    extra_tokens: int               # always-present fusion tokens at the end
    d: int
    Hq: int
    Hk: int
    dh: int
    F: int
    n_layers: int
    head_keep: object               # float, or (lo, hi) drawn per layer
    ffn_keep: float
    dropout: str                    # "none" | "last" | "bernoulli:p" | "upto:k"
    final_ln: bool
    seed: int
    c: int = 5
    act: int = 0                    # 0 ReLU, 1 erf-GELU

    @property
    def M(self) -> int:
        return len(self.seg_tokens)

    @property
    def L(self) -> int:
        return int(sum(self.seg_tokens)) + self.extra_tokens


CONFIGS: Dict[str, Spec] = {
    # tiny single layer, fp32; modality 3 dropped for every sample
    "C1": Spec("C1", "f32", 2, (16, 16, 16), 0, 64, 4, 2, 16, 256, 1, 0.5, 0.5, "last", False, 0),
    # single layer, bf16 in / fp32 accumulate; Bernoulli(0.3) modality dropout
    "C2": Spec("C2", "bf16", 64, (128, 128, 128), 0, 256, 8, 2, 32, 1024, 1, 0.75, 0.6,
               "bernoulli:0.3", False, 2000),
    # four modalities at different rates; 0-2 modalities dropped per sample
    "C3": Spec("C3", "bf16", 256, (256, 128, 64, 32), 0, 512, 8, 4, 64, 2048, 1, 0.5, 0.5,
               "upto:2", False, 3000),
    # 6-layer pre-norm stack, 3 x 170 tokens + 2 fusion tokens
    "C4": Spec("C4", "bf16", 128, (170, 170, 170), 2, 512, 8, 2, 64, 2048, 6, (0.6, 0.9), 0.6,
               "none", True, 4000),
    # long-sequence stress layer
    "C5": Spec("C5", "bf16", 16, (2048, 2048), 0, 768, 12, 4, 64, 3072, 1, 0.7, 0.7,
               "none", False, 5000),
}


@dataclass
class Workload:
    spec: Spec
    x: np.ndarray                       # [B, L, d] fp32 (bf16-valued when spec.dtype == "bf16")
    presence: np.ndarray                # [B, M] uint8; which positions a sample may attend to follows from it and
    tok_modality: np.ndarray            # [L] int32, -1 = always present - derived by the library and by the oracle, each on its own
    pattern_bits: np.ndarray            # [P] presence bit patterns in use (ascending)
    pattern_id: np.ndarray              # [B] int32 index into pattern_bits
    g_head: np.ndarray                  # [nl, P, Hq] fp32 gate scores
    g_ffn: np.ndarray                   # [nl, P, F]
    k_head: np.ndarray                  # [nl] int32
    k_ffn: np.ndarray                   # [nl] int32
    layers: List[Dict[str, np.ndarray]] = field(default_factory=list)   # dense weights per layer
    final_ln: Optional[Dict[str, np.ndarray]] = None

    @property
    def P(self) -> int:
        return int(self.pattern_bits.shape[0])


def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, tensor_id]))


def _presence(spec: Spec, B: int, rng: np.random.Generator) -> np.ndarray:
    M = spec.M
    pres = np.ones((B, M), dtype=np.uint8)
    kind = spec.dropout
    if kind == "none":
        return pres
    if kind == "last":
        pres[:, M - 1] = 0
        return pres
    if kind.startswith("bernoulli:"):
        p = float(kind.split(":")[1])
        for b in range(B):
            while True:
                row = (rng.random(M) >= p).astype(np.uint8)
                if row.any():
                    break
            pres[b] = row
        return pres
    if kind.startswith("upto:"):
        kmax = int(kind.split(":")[1])
        for b in range(B):
            n_drop = int(rng.integers(0, kmax + 1))
            drop = rng.choice(M, size=n_drop, replace=False)
            pres[b, drop] = 0
        return pres
    raise ValueError(kind)


def make_workload(spec: Spec, B: Optional[int] = None, affine_noise: bool = True,
                  with_x: bool = True) -> Workload:
    """Draw every tensor of a workload.

    Activations N(0,1); weight matrices N(0, 1/fan_in) (std = 1/sqrt(fan_in));
    biases N(0, 0.02^2); LayerNorm gamma = 1 + N(0, 0.05^2), beta N(0, 0.05^2)
    (exactly 1 / 0 with affine_noise=False); gate scores U(0,1) drawn for all
    2^M presence patterns, of which only the patterns in use are kept.
    B overrides the batch (the first B samples of the same random streams are
    NOT guaranteed identical; a smaller B is its own workload).
    """
    B = spec.B if B is None else int(B)
    L, d, M = spec.L, spec.d, spec.M
    Hq, Hk, dh, F, nl = spec.Hq, spec.Hk, spec.dh, spec.F, spec.n_layers
    q = storage_rounding(spec.dtype)
    seed = spec.seed

    tok_mod = np.concatenate(
        [np.full(n, m, dtype=np.int32) for m, n in enumerate(spec.seg_tokens)]
        + [np.full(spec.extra_tokens, -1, dtype=np.int32)])
    presence = _presence(spec, B, _rng(seed, 1))
    bits = (presence.astype(np.int64) << np.arange(M)).sum(axis=1)
    pattern_bits = np.unique(bits)
    pattern_id = np.searchsorted(pattern_bits, bits).astype(np.int32)

    x = q(_rng(seed, 2).standard_normal((B, L, d), dtype=np.float32)) if with_x else np.zeros((0, L, d), np.float32)

    g_head_all = _rng(seed, 3).random((nl, 2 ** M, Hq), dtype=np.float32)
    g_ffn_all = _rng(seed, 4).random((nl, 2 ** M, F), dtype=np.float32)
    g_head = np.ascontiguousarray(g_head_all[:, pattern_bits, :])
    g_ffn = np.ascontiguousarray(g_ffn_all[:, pattern_bits, :])

    if isinstance(spec.head_keep, tuple):
        lo, hi = spec.head_keep
        ratios = _rng(seed, 5).uniform(lo, hi, size=nl)
    else:
        ratios = np.full(nl, float(spec.head_keep))
    k_head = np.array([keep_count(float(r), Hq) for r in ratios], dtype=np.int32)
    k_ffn = np.full(nl, keep_count(spec.ffn_keep, F), dtype=np.int32)

    def mat(rng, rows, cols, fan_in):
        return q(rng.standard_normal((rows, cols), dtype=np.float32) / np.float32(math.sqrt(fan_in)))

    def vec(rng, n, std, base=0.0, ln=False):
        if ln and not affine_noise:
            return q(np.full(n, base, dtype=np.float32))
        return q(np.float32(base) + np.float32(std) * rng.standard_normal(n, dtype=np.float32))

    layers = []
    for l in range(nl):
        r = _rng(seed, 100 + l)
        layers.append({
            "Wq": mat(r, Hq * dh, d, d), "bq": vec(r, Hq * dh, 0.02),
            "Wk": mat(r, Hk * dh, d, d), "bk": vec(r, Hk * dh, 0.02),
            "Wv": mat(r, Hk * dh, d, d), "bv": vec(r, Hk * dh, 0.02),
            "Wo": mat(r, Hq * dh, d, Hq * dh), "bo": vec(r, d, 0.02),
            "W1": mat(r, F, d, d), "b1": vec(r, F, 0.02),
            "W2": mat(r, F, d, F), "b2": vec(r, d, 0.02),
            "ln1_g": vec(r, d, 0.05, 1.0, True), "ln1_b": vec(r, d, 0.05, 0.0, True),
            "ln2_g": vec(r, d, 0.05, 1.0, True), "ln2_b": vec(r, d, 0.05, 0.0, True),
        })
    final_ln = None
    if spec.final_ln:
        r = _rng(seed, 99)
        final_ln = {"g": vec(r, d, 0.05, 1.0, True), "b": vec(r, d, 0.05, 0.0, True)}

    return Workload(spec, x, presence, tok_mod, pattern_bits, pattern_id,
                    g_head, g_ffn, k_head, k_ffn, layers, final_ln)


def small_spec(name: str = "S", dtype: str = "f32", B: int = 3, seg=(7, 5, 9), extra: int = 1,
               d: int = 32, Hq: int = 4, Hk: int = 2, dh: int = 8, F: int = 48, nl: int = 2,
               head_keep=0.5, ffn_keep: float = 0.5, dropout: str = "bernoulli:0.3",
               final_ln: bool = True, seed: int = 7, c: int = 2, act: int = 0) -> Spec:
    """A free-form small spec for tests (ragged sizes, several patterns)."""
    return Spec(name, dtype, B, tuple(seg), extra, d, Hq, Hk, dh, F, nl, head_keep, ffn_keep,
                dropout, final_ln, seed, c, act)


@dataclass
class MoeBlock:
    """A Sparse-MoE FFN block on top of a workload's tokens: E experts with their own gate scores and
    keep counts (ragged F'_e), a router, Top-k.  Arrays are fp32 holding values of the workload's dtype."""
    E: int
    top_k: int
    dense: Dict[str, np.ndarray]        # Wr [E,d], br [E], W1 [E,F,d], b1 [E,F], W2 [E,F,d], b2 [E,d], ln_g, ln_b [d]
    g_ffn: np.ndarray                   # [E, P, F] expert-internal gate scores per pattern in use
    k_ffn: np.ndarray                   # [E] kept channels per expert


def make_moe_block(wl: Workload, E: int, top_k: int, keep=(0.4, 0.8), seed_offset: int = 500) -> MoeBlock:
    """Seeded MoE block for the tokens of `wl` (same d, F, patterns).  Router rows N(0, 1/d) so that the
    logits are O(1); expert weights as the FFN of make_workload; keep ratios U(keep) per expert."""
    spec = wl.spec
    d, F, M = spec.d, spec.F, spec.M
    q = storage_rounding(spec.dtype)
    r = _rng(spec.seed, seed_offset)
    sd, sF = np.float32(1.0 / math.sqrt(d)), np.float32(1.0 / math.sqrt(F))
    dense = {
        "Wr": q(r.standard_normal((E, d), dtype=np.float32) * sd),
        "br": q(np.float32(0.02) * r.standard_normal(E, dtype=np.float32)),
        "W1": q(r.standard_normal((E, F, d), dtype=np.float32) * sd),
        "b1": q(np.float32(0.02) * r.standard_normal((E, F), dtype=np.float32)),
        "W2": q(r.standard_normal((E, F, d), dtype=np.float32) * sF),
        "b2": q(np.float32(0.02) * r.standard_normal((E, d), dtype=np.float32)),
        "ln_g": q(np.float32(1.0) + np.float32(0.05) * r.standard_normal(d, dtype=np.float32)),
        "ln_b": q(np.float32(0.05) * r.standard_normal(d, dtype=np.float32)),
    }
    g_all = r.random((E, 2 ** M, F), dtype=np.float32)
    g_ffn = np.ascontiguousarray(g_all[:, wl.pattern_bits, :])
    lo, hi = keep
    k_ffn = np.array([keep_count(float(x), F) for x in r.uniform(lo, hi, size=E)], dtype=np.int32)
    return MoeBlock(E, top_k, dense, g_ffn, k_ffn)


def make_gate_params(nl: int, M: int, Hq: int, F: int, Hd: int = 16, seed: int = 0, seed_offset: int = 900) -> Dict[str, np.ndarray]:
    """Seeded parameters of the gating module of Eq. (1), fp32: a first layer shared per layer (Wa [nl,Hd,M],
    ba [nl,Hd]), one output row per unit (Wb [nl,Hq+F,Hd], cb), base importances zeta ~ N(0,1) and a per-layer
    scale gamma ~ U(0.5, 2).  Stands in for a trained gate by shape only."""
    r = _rng(seed, seed_offset)
    n = Hq + F
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    return {"Wa": f32(r.standard_normal((nl, Hd, M))), "ba": f32(0.3 * r.standard_normal((nl, Hd))),
            "Wb": f32(r.standard_normal((nl, n, Hd)) / math.sqrt(Hd)), "cb": f32(0.2 * r.standard_normal((nl, n))),
            "zeta": f32(r.standard_normal((nl, n))), "gamma": f32(r.uniform(0.5, 2.0, nl))}


def unit_costs(spec: Spec, U: int):
    """Integer cost table for the budget search: multiply-adds x 2 per sample of one kept head (Q and output
    projection, score stream, active rows), one kept K/V group (K and V projection) and one kept FFN channel
    (both FFN matrices), per layer.  Plain shape arithmetic of the dense operators; not part of the method."""
    L, d, dh = spec.L, spec.d, spec.dh
    head = 2 * L * d * dh * 2 + (2 * L * L * dh if 0 < U < L else 0) + 4 * min(U, L) * L * dh
    group = 2 * L * d * dh * 2
    ffn = 4 * L * d
    nl = spec.n_layers
    return [head] * nl, [group] * nl, [ffn] * nl
