"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It loads (and, if needed, compiles with gcc) oracle/sentry_oracle.c
and marshals numpy arrays; it contains no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sentry_oracle.c")
_LIB = os.path.join(_HERE, "libsentry_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "sentry_oracle.h"))):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class _Layer(C.Structure):
    _fields_ = ([("nH", C.c_int32), ("nG", C.c_int32), ("dh", C.c_int32), ("d", C.c_int32),
                 ("F", C.c_int32)]
                + [(n, C.c_void_p) for n in ("Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo",
                                             "W1", "b1", "W2", "b2",
                                             "ln1_g", "ln1_b", "ln2_g", "ln2_b",
                                             "head_group", "head_mask", "ffn_mask")])


class _Moe(C.Structure):
    _fields_ = ([("d", C.c_int32), ("F", C.c_int32), ("E", C.c_int32), ("k", C.c_int32)]
                + [(n, C.c_void_p) for n in ("Wr", "br", "W1", "b1", "W2", "b2", "ffn_mask", "ln_g", "ln_b")])


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_num_active.restype = C.c_int32
        _lib.orc_round_bf16.restype = C.c_double
        _lib.orc_round_bf16.argtypes = [C.c_double]
        _lib.orc_round_f16.restype = C.c_double
        _lib.orc_round_f16.argtypes = [C.c_double]
        _lib.orc_max_threads.restype = C.c_int32
        _lib.orc_fp8_e4m3_decode.restype = C.c_double
        _lib.orc_fp8_e4m3_encode.restype = C.c_uint8
        _lib.orc_f16_decode.restype = C.c_double
        _lib.orc_dequant_f16.restype = None
        _lib.orc_pruned_ffn_fp8.restype = None
        _lib.orc_quantize_fp8.restype = None
        _lib.orc_fp8_e4m3_decode.argtypes = [C.c_uint8]
        for f in ("orc_key_valid", "orc_gate_scores_to_masks", "orc_sparse_gqa", "orc_encoder_forward", "orc_encoder_forward_fp8ffn", "orc_encoder_forward_fp8", "orc_moe_ffn",
                  "orc_gate_eval", "orc_budget_search"):
            getattr(_lib, f).restype = C.c_int32
    return _lib


class _Ffn8(C.Structure):
    _fields_ = [("W1q", C.c_void_p), ("W2q", C.c_void_p), ("s1", C.c_float), ("s2", C.c_float), ("sx", C.c_float),
                ("sh", C.c_float)]


class _Proj8(C.Structure):
    _fields_ = [("Wq8", C.c_void_p), ("Wk8", C.c_void_p), ("Wv8", C.c_void_p), ("Wo8", C.c_void_p),
                ("s_qkv", C.c_float), ("so", C.c_float), ("sx1", C.c_float), ("sa", C.c_float)]


class _Fp8Io(C.Structure):
    _fields_ = ([(n, C.c_void_p) for n in ("xq_forced", "hq_forced", "aq_forced", "oq_forced")]
                + [(n, C.c_int32) for n in ("n_forced_x", "n_forced_h", "n_forced_a", "n_forced_o")]
                + [(n, C.c_void_p) for n in ("xq_out", "hq_out", "aq_out", "oq_out")])


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def max_threads() -> int:
    return int(lib().orc_max_threads())


def num_active(T: int, c: int) -> int:
    return int(lib().orc_num_active(C.c_int32(T), C.c_int32(c)))


def round_bf16(a) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    out = np.empty_like(a)
    f = lib().orc_round_bf16
    flat_in, flat_out = a.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = f(float(flat_in[i]))
    return out


def round_f16(a) -> np.ndarray:
    """nearest IEEE binary16 values.  Functions that take `bf16` accept 0 / False (no storage rounding), 1 / True
    (bfloat16) and 2 (binary16, the FP16 variant of the model)."""
    a = np.asarray(a, dtype=np.float64)
    out = np.empty_like(a)
    f = lib().orc_round_f16
    flat_in, flat_out = a.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = f(float(flat_in[i]))
    return out


def key_valid(presence, tok_modality) -> np.ndarray:
    """[B, L] uint8: which positions of the token sequence sample b may use as keys (Sec. 4.2 / 4.4)."""
    pres = np.ascontiguousarray(presence, dtype=np.uint8)
    tm = np.ascontiguousarray(tok_modality, dtype=np.int32)
    B, M = pres.shape
    out = np.empty((B, tm.shape[0]), np.uint8)
    rc = lib().orc_key_valid(B, M, tm.shape[0], _p(pres), _p(tm), _p(out))
    if rc != 0:
        raise ValueError(f"orc_key_valid: status {rc}")
    return out


def gate_scores_to_masks(g_head, g_ffn, k_head, k_ffn, Hk: int) -> Dict[str, np.ndarray]:
    g_head = np.ascontiguousarray(g_head, dtype=np.float32)
    g_ffn = np.ascontiguousarray(g_ffn, dtype=np.float32)
    nl, P, Hq = g_head.shape
    F = g_ffn.shape[2]
    k_head = np.ascontiguousarray(k_head, dtype=np.int32)
    k_ffn = np.ascontiguousarray(k_ffn, dtype=np.int32)
    out = {
        "head_mask": np.zeros((nl, P, Hq), np.uint8), "ffn_mask": np.zeros((nl, P, F), np.uint8),
        "head_idx": np.zeros((nl, P, Hq), np.int32), "ffn_idx": np.zeros((nl, P, F), np.int32),
        "group_idx": np.zeros((nl, P, Hk), np.int32), "n_groups": np.zeros((nl, P), np.int32),
        "head_group": np.zeros((nl, P, Hq), np.int32),
    }
    rc = lib().orc_gate_scores_to_masks(
        C.c_int32(nl), C.c_int32(P), C.c_int32(Hq), C.c_int32(Hk), C.c_int32(F),
        _p(g_head), _p(g_ffn), _p(k_head), _p(k_ffn),
        _p(out["head_mask"]), _p(out["ffn_mask"]), _p(out["head_idx"]), _p(out["ffn_idx"]),
        _p(out["group_idx"]), _p(out["n_groups"]), _p(out["head_group"]))
    if rc != 0:
        raise ValueError("orc_gate_scores_to_masks: bad arguments")
    return out


def gather_rows(src, idx, block: int = 1) -> np.ndarray:
    src = _f64(src)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    row_len = int(np.prod(src.shape[1:])) if src.ndim > 1 else 1
    dst = np.zeros((idx.size * block,) + src.shape[1:], np.float64)
    lib().orc_gather_rows(_p(src), _p(idx), C.c_int32(idx.size), C.c_int32(block),
                          C.c_int64(row_len), _p(dst))
    return dst


def layernorm(x, gamma, beta, eps: float = 1e-5, bf16: bool = False) -> np.ndarray:
    x = _f64(x)
    d = x.shape[-1]
    y = np.empty_like(x)
    g, b = _f64(gamma), _f64(beta)
    lib().orc_layernorm(_p(x), C.c_int64(x.size // d), C.c_int32(d), _p(g), _p(b),
                        C.c_double(eps), C.c_int32(int(bf16)), _p(y))
    return y


def _sample(sample_idx, B):
    if sample_idx is None:
        return None, 0
    si = np.ascontiguousarray(sample_idx, dtype=np.int32)
    assert si.ndim == 2 and si.shape[0] == B, si.shape
    return si, si.shape[1]


def sparse_gqa(Q, K, V, head_group, U: int, key_valid=None, forced_sel=None, bf16: bool = False,
               head_group_b=None, want_score: bool = True, sample_idx=None):
    """Returns (O [B,L,nH*dh], score [B,nH,L], sel [B,nH,U], prob_check [2]).
    sample_idx [B,S] (optional): key sample of the sparsity score."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, nH, L, dh = Q.shape
    nG = K.shape[1]
    assert K.shape == (B, nG, L, dh) and V.shape == K.shape
    hg = np.ascontiguousarray(head_group, dtype=np.int32)
    hgb = None if head_group_b is None else np.ascontiguousarray(head_group_b, dtype=np.int32)
    kv = None if key_valid is None else np.ascontiguousarray(key_valid, dtype=np.uint8)
    fs = None if forced_sel is None else np.ascontiguousarray(forced_sel, dtype=np.int32)
    O = np.zeros((B, L, nH * dh), np.float64)
    score = np.zeros((B, nH, L), np.float64) if want_score else None
    sel = np.full((B, nH, max(U, 1)), -1, np.int32)
    chk = np.zeros(2, np.float64)
    si, ns = _sample(sample_idx, B)
    rc = lib().orc_sparse_gqa(C.c_int32(B), C.c_int32(nH), C.c_int32(nG), C.c_int32(L),
                              C.c_int32(dh), _p(Q), _p(K), _p(V), _p(hg), _p(hgb), _p(kv),
                              _p(si), C.c_int32(ns),
                              C.c_int32(U), _p(fs), C.c_int32(int(bf16)), _p(O), _p(score),
                              _p(sel), _p(chk))
    if rc != 0:
        raise ValueError("orc_sparse_gqa: bad arguments")
    return O, score, sel[:, :, :U], chk


class LayerPack:
    """Keeps the float64 copies alive for as long as the C struct is used."""

    def __init__(self, w: Dict[str, np.ndarray], nH: int, nG: int, dh: int, head_group,
                 head_mask=None, ffn_mask=None):
        self.keep = {}
        s = _Layer()
        d = int(np.asarray(w["Wq"]).shape[1])
        F = int(np.asarray(w["W1"]).shape[0])
        s.nH, s.nG, s.dh, s.d, s.F = nH, nG, dh, d, F
        assert np.asarray(w["Wq"]).shape == (nH * dh, d), (np.asarray(w["Wq"]).shape, nH, dh, d)
        assert np.asarray(w["Wk"]).shape == (nG * dh, d)
        assert np.asarray(w["Wo"]).shape == (nH * dh, d)
        assert np.asarray(w["W2"]).shape == (F, d)
        for n in ("Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo", "W1", "b1", "W2", "b2",
                  "ln1_g", "ln1_b", "ln2_g", "ln2_b"):
            a = _f64(w.get(n))
            self.keep[n] = a
            setattr(s, n, None if a is None else a.ctypes.data)
        hg = np.ascontiguousarray(head_group, dtype=np.int32)
        assert hg.shape == (nH,)
        hm = None if head_mask is None else np.ascontiguousarray(head_mask, dtype=np.uint8)
        fm = None if ffn_mask is None else np.ascontiguousarray(ffn_mask, dtype=np.uint8)
        self.keep.update(hg=hg, hm=hm, fm=fm)
        s.head_group = hg.ctypes.data
        s.head_mask = None if hm is None else hm.ctypes.data
        s.ffn_mask = None if fm is None else fm.ctypes.data
        self.struct = s


def pruned_ffn(pack: LayerPack, x, act: int = 0, eps: float = 1e-5, pre_ln: bool = True,
               add_residual: bool = True, bf16: bool = False) -> np.ndarray:
    x = _f64(x)
    d = x.shape[-1]
    y = np.empty_like(x)
    lib().orc_pruned_ffn(C.byref(pack.struct), _p(x), C.c_int64(x.size // d), C.c_int32(act),
                         C.c_double(eps), C.c_int32(int(pre_ln)), C.c_int32(int(add_residual)),
                         C.c_int32(int(bf16)), _p(y))
    return y


def moe_ffn(x, moe: Dict[str, np.ndarray], top_k: int, act: int = 0, eps: float = 1e-5, pre_ln: bool = True,
            add_residual: bool = True, bf16: bool = False, ffn_mask=None, forced_route=None):
    """Sparse-MoE FFN of one presence pattern.  moe: Wr [E,d], br [E] | None, W1 [E,F,d], b1 [E,F] | None,
    W2 [E,F,d], b2 [E,d] | None, ln_g, ln_b [d].  ffn_mask [E,F] u8 (1 = kept) or None.
    Returns (y [rows,d], route [rows,k], weight [rows,k], logit [rows,E])."""
    x = _f64(x)
    d = x.shape[-1]
    rows = x.size // d
    keep = {k: _f64(moe.get(k)) for k in ("Wr", "br", "W1", "b1", "W2", "b2", "ln_g", "ln_b")}
    E, F = keep["W1"].shape[0], keep["W1"].shape[1]
    assert keep["Wr"].shape == (E, d) and keep["W2"].shape == (E, F, d)
    fm = None if ffn_mask is None else np.ascontiguousarray(ffn_mask, dtype=np.uint8)
    fr = None if forced_route is None else np.ascontiguousarray(forced_route, dtype=np.int32)
    st = _Moe(d, F, E, top_k, *[_p(keep[k]) for k in ("Wr", "br", "W1", "b1", "W2", "b2")], _p(fm),
              _p(keep["ln_g"]), _p(keep["ln_b"]))
    y = np.empty_like(x)
    route = np.full((rows, top_k), -1, np.int32)
    weight = np.zeros((rows, top_k), np.float64)
    logit = np.zeros((rows, E), np.float64)
    rc = lib().orc_moe_ffn(C.byref(st), _p(x), C.c_int64(rows), C.c_int32(act), C.c_double(eps),
                           C.c_int32(int(pre_ln)), C.c_int32(int(add_residual)), C.c_int32(int(bf16)), _p(fr),
                           _p(y), _p(route), _p(weight), _p(logit))
    if rc != 0:
        raise ValueError("orc_moe_ffn: bad arguments")
    return y, route, weight, logit


def gate_eval(gate: Dict[str, np.ndarray], pattern_bits, Hq: int, nonlin: int = 0):
    """Eq. (1) for every layer and presence pattern.  gate: Wa [nl,Hd,M], ba [nl,Hd], Wb [nl,Hq+F,Hd],
    cb [nl,Hq+F], zeta [nl,Hq+F], gamma [nl].  Returns (g_head [nl,P,Hq], g_ffn [nl,P,F]) in fp64."""
    Wa, ba, Wb, cb, zeta = (_f64(gate[k]) for k in ("Wa", "ba", "Wb", "cb", "zeta"))
    gamma = _f64(gate["gamma"])
    nl, Hd, M = Wa.shape
    n_units = Wb.shape[1]
    bits = np.asarray(pattern_bits, dtype=np.int64)
    out = np.empty((nl, len(bits), n_units), np.float64)
    row = np.empty(n_units, np.float64)
    for l in range(nl):
        for p, b in enumerate(bits):
            rc = lib().orc_gate_eval(C.c_int32(M), C.c_int32(Hd), C.c_int32(n_units), C.c_int32(nonlin),
                                     _p(Wa[l]), _p(ba[l]), _p(Wb[l]), _p(cb[l]), _p(zeta[l]),
                                     C.c_double(float(gamma[l])), C.c_uint32(int(b)), _p(row))
            if rc != 0:
                raise ValueError("orc_gate_eval: bad arguments")
            out[l, p] = row
    return np.ascontiguousarray(out[:, :, :Hq]), np.ascontiguousarray(out[:, :, Hq:])


def budget_search(g_head, g_ffn, Hk: int, c_head, c_group, c_ffn, c_fixed: int, budget: int):
    """g_head [nl,Hq], g_ffn [nl,F] fp32 scores of one pattern.  Returns dict(feasible, tau, k_head, k_ffn, cost)."""
    g_head = np.ascontiguousarray(g_head, dtype=np.float32)
    g_ffn = np.ascontiguousarray(g_ffn, dtype=np.float32)
    nl, Hq = g_head.shape
    F = g_ffn.shape[1]
    ch, cg, cf = (np.ascontiguousarray(a, dtype=np.int64) for a in (c_head, c_group, c_ffn))
    assert ch.shape == (nl,) and cg.shape == (nl,) and cf.shape == (nl,)
    tau, cost = C.c_float(0.0), C.c_int64(0)
    k_head, k_ffn = np.zeros(nl, np.int32), np.zeros(nl, np.int32)
    rc = lib().orc_budget_search(C.c_int32(nl), C.c_int32(Hq), C.c_int32(Hk), C.c_int32(F), _p(g_head), _p(g_ffn),
                                 _p(ch), _p(cg), _p(cf), C.c_int64(int(c_fixed)), C.c_int64(int(budget)),
                                 C.byref(tau), _p(k_head), _p(k_ffn), C.byref(cost))
    if rc < 0:
        raise ValueError("orc_budget_search: bad arguments")
    return {"feasible": bool(rc), "tau": np.float32(tau.value), "k_head": k_head, "k_ffn": k_ffn, "cost": int(cost.value)}


def fp8_e4m3_decode(b: int) -> float:
    return float(lib().orc_fp8_e4m3_decode(C.c_uint8(int(b))))


def dequant_fp8(q, scale: float, bf16: bool) -> np.ndarray:
    """q uint8 (OCP E4M3 codes) -> decode(q) * scale rounded to the model dtype, as fp64."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    out = np.empty(q.shape, np.float64)
    lib().orc_dequant_fp8(_p(q), C.c_int64(q.size), C.c_float(float(scale)), C.c_int32(int(bf16)), _p(out))
    return out


def f16_decode(bits: int) -> float:
    return float(lib().orc_f16_decode(C.c_uint16(int(bits))))


def dequant_f16(q, bf16: bool) -> np.ndarray:
    """q uint16 (IEEE binary16 bit patterns) -> their values rounded to the model dtype, as fp64."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    out = np.empty(q.shape, np.float64)
    lib().orc_dequant_f16(_p(q), C.c_int64(q.size), C.c_int32(int(bf16)), _p(out))
    return out


def fp8_e4m3_encode(t: float) -> int:
    return int(lib().orc_fp8_e4m3_encode(C.c_float(float(t))))


def quantize_fp8(x, scale: float) -> np.ndarray:
    """x (taken as fp32) -> E4M3 codes of fl32(x * fl32(1/scale)), ties to even, saturating at +-448."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, np.uint8)
    lib().orc_quantize_fp8(_p(x), C.c_int64(x.size), C.c_float(float(scale)), _p(out))
    return out


def pruned_ffn_fp8(x, W1q, s1: float, b1, W2q, s2: float, b2, ln_g, ln_b, sx: float, sh: float, ffn_mask=None,
                   act: int = 0, eps: float = 1e-5, pre_ln: bool = True, add_residual: bool = True,
                   bf16: bool = True, xq_forced=None, hq_forced=None, want_z: bool = False):
    """FFN block in FP8 arithmetic (see orc_pruned_ffn_fp8).  W1q, W2q [F,d] uint8 codes (dense layout).
    xq_forced [rows,d] / hq_forced [rows,F]: codes to use instead of the block's own.
    Returns (y [rows,d] fp64, xq [rows,d] uint8, hq [rows,F] uint8) and, with want_z, z [rows,F]."""
    x = _f64(x)
    d = x.shape[-1]
    rows = x.size // d
    W1q = np.ascontiguousarray(W1q, dtype=np.uint8)
    W2q = np.ascontiguousarray(W2q, dtype=np.uint8)
    F = W1q.shape[0]
    assert W1q.shape == (F, d) and W2q.shape == (F, d)
    b1, b2, ln_g, ln_b = _f64(b1), _f64(b2), _f64(ln_g), _f64(ln_b)
    fm = None if ffn_mask is None else np.ascontiguousarray(ffn_mask, dtype=np.uint8)
    y = np.empty_like(x)
    xq = np.empty((rows, d), np.uint8)
    hq = np.empty((rows, F), np.uint8)
    xf = None if xq_forced is None else np.ascontiguousarray(xq_forced, dtype=np.uint8).reshape(rows, d)
    hf = None if hq_forced is None else np.ascontiguousarray(hq_forced, dtype=np.uint8).reshape(rows, F)
    z = np.empty((rows, F), np.float64) if want_z else None
    lib().orc_pruned_ffn_fp8(C.c_int32(d), C.c_int32(F), _p(W1q), C.c_float(float(s1)), _p(b1), _p(W2q),
                             C.c_float(float(s2)), _p(b2), _p(ln_g), _p(ln_b), _p(fm), C.c_float(float(sx)),
                             C.c_float(float(sh)), _p(x), C.c_int64(rows), C.c_int32(act), C.c_double(eps),
                             C.c_int32(int(pre_ln)), C.c_int32(int(add_residual)), C.c_int32(int(bf16)), _p(xf),
                             _p(hf), _p(y), _p(xq), _p(hq), _p(z))
    return (y, xq, hq, z) if want_z else (y, xq, hq)


def encoder_forward(x, packs: Sequence[Sequence[LayerPack]], U: int, pattern_id=None,
                    key_valid=None, act: int = 0, eps: float = 1e-5, forced_sel=None,
                    final_ln: Optional[Dict[str, np.ndarray]] = None, bf16: bool = False,
                    want_sel: bool = True, want_score: bool = False, sample_idx=None, ffn8=None, xq_forced=None,
                    hq_forced=None, want_codes: bool = False, n_forced_x=None, n_forced_h=None, proj8=None,
                    aq_forced=None, oq_forced=None, n_forced_a=None, n_forced_o=None):
    """packs[l][p] = LayerPack of layer l, pattern p.
    ffn8: per layer a dict W1q, W2q [F,d] uint8, s1, s2, sx, sh - the layer's FFN runs in FP8 arithmetic;
    xq_forced [nl,B,L,d], hq_forced [nl,B,L,F] uint8: codes to use instead of the oracle's own, in the layers
    l < n_forced_x / l < n_forced_h (default: every layer).
    proj8: per layer a dict Wq8 [nH*dh,d], Wk8, Wv8 [nG*dh,d], Wo8 [nH*dh,d] uint8, s_qkv, so, sx1, sa - the
    layer's Q/K/V and output projections run in FP8 arithmetic; aq_forced [nl,B,L,d] (codes of LN1(x)) and
    oq_forced [nl,B,L,nH*dh] (codes of the attention output) work like xq_forced.
    Returns (y [B,L,d], sel [nl,B,nHmax,U] or None, score [nl,B,nHmax,L] or None) and, with want_codes,
    xq [nl,B,L,d], hq [nl,B,L,F] (None without ffn8) and, with proj8, aq [nl,B,L,d], oq [nl,B,L,nH*dh]."""
    x = _f64(x)
    B, L, d = x.shape
    nl, P = len(packs), len(packs[0])
    arr = (_Layer * (nl * P))()
    nHmax = 0
    for l in range(nl):
        for p in range(P):
            arr[l * P + p] = packs[l][p].struct
            nHmax = max(nHmax, packs[l][p].struct.nH)
    pid = None if pattern_id is None else np.ascontiguousarray(pattern_id, dtype=np.int32)
    kv = None if key_valid is None else np.ascontiguousarray(key_valid, dtype=np.uint8)
    fs = None
    if forced_sel is not None:
        fs = np.ascontiguousarray(forced_sel, dtype=np.int32)
        assert fs.shape == (nl, B, nHmax, U), (fs.shape, (nl, B, nHmax, U))
    fg = None if final_ln is None else _f64(final_ln["g"])
    fb = None if final_ln is None else _f64(final_ln["b"])
    y = np.empty_like(x)
    sel = np.full((nl, B, nHmax, max(U, 1)), -1, np.int32) if want_sel else None
    score = np.full((nl, B, nHmax, L), -np.inf, np.float64) if want_score else None
    si, ns = _sample(sample_idx, B)
    f8 = p8 = xf = hf = af = of = xq = hq = aq = oq = None
    keep8 = []
    F = packs[0][0].struct.F
    nH, dh, nG = packs[0][0].struct.nH, packs[0][0].struct.dh, packs[0][0].struct.nG
    if ffn8 is not None:
        assert len(ffn8) == nl
        f8 = (_Ffn8 * nl)()
        for l, f in enumerate(ffn8):
            a, b = np.ascontiguousarray(f["W1q"], dtype=np.uint8), np.ascontiguousarray(f["W2q"], dtype=np.uint8)
            assert a.shape == (F, d) and b.shape == (F, d)
            keep8 += [a, b]
            f8[l] = _Ffn8(_p(a), _p(b), float(f["s1"]), float(f["s2"]), float(f["sx"]), float(f["sh"]))
        if xq_forced is not None:
            xf = np.ascontiguousarray(xq_forced, dtype=np.uint8).reshape(nl, B, L, d)
        if hq_forced is not None:
            hf = np.ascontiguousarray(hq_forced, dtype=np.uint8).reshape(nl, B, L, F)
        if want_codes:
            xq, hq = np.empty((nl, B, L, d), np.uint8), np.empty((nl, B, L, F), np.uint8)
    if proj8 is not None:
        assert len(proj8) == nl and nH == nHmax
        p8 = (_Proj8 * nl)()
        for l, f in enumerate(proj8):
            ws = [np.ascontiguousarray(f[k], dtype=np.uint8) for k in ("Wq8", "Wk8", "Wv8", "Wo8")]
            assert ws[0].shape == (nH * dh, d) and ws[1].shape == (nG * dh, d) and ws[2].shape == (nG * dh, d)
            assert ws[3].shape == (nH * dh, d)
            keep8 += ws
            p8[l] = _Proj8(_p(ws[0]), _p(ws[1]), _p(ws[2]), _p(ws[3]), float(f["s_qkv"]), float(f["so"]),
                           float(f["sx1"]), float(f["sa"]))
        if aq_forced is not None:
            af = np.ascontiguousarray(aq_forced, dtype=np.uint8).reshape(nl, B, L, d)
        if oq_forced is not None:
            of = np.ascontiguousarray(oq_forced, dtype=np.uint8).reshape(nl, B, L, nH * dh)
        if want_codes:
            aq, oq = np.empty((nl, B, L, d), np.uint8), np.empty((nl, B, L, nH * dh), np.uint8)

    def cnt(v):
        return nl if v is None else int(v)

    io = _Fp8Io(_p(xf), _p(hf), _p(af), _p(of), cnt(n_forced_x), cnt(n_forced_h), cnt(n_forced_a), cnt(n_forced_o),
                _p(xq), _p(hq), _p(aq), _p(oq))
    rc = lib().orc_encoder_forward_fp8(
        C.c_int32(B), C.c_int32(L), C.c_int32(nl), C.c_int32(P), arr, f8, p8, _p(pid), _p(kv),
        _p(si), C.c_int32(ns), C.c_int32(U), C.c_int32(act), C.c_double(eps), _p(fs), C.c_int32(nHmax), _p(fg), _p(fb),
        C.c_int32(int(bf16)), C.byref(io), _p(x), _p(y), _p(sel), _p(score))
    if rc != 0:
        raise ValueError("orc_encoder_forward: bad arguments")
    if sel is not None:
        sel = sel[..., :U]
    if not want_codes:
        return y, sel, score
    return (y, sel, score, xq, hq, aq, oq) if proj8 is not None else (y, sel, score, xq, hq)
