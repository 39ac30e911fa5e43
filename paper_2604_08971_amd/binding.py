"""Thin ctypes binding of libsentryfuse.so (the gfx950 HIP library).

Argument marshalling only: every step of the path runs in the library's
kernels.  PyTorch is used for device memory and the current HIP stream.
There is no CPU fallback: if the shared library has not been built, loading
raises.
"""
from __future__ import annotations

import contextlib
import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsentryfuse.so")
# the build of the same sources whose 16-bit type is IEEE binary16 (dtype SF_F16); selected with use_half("f16")
LIB_PATHS = {"bf16": LIB_PATH, "f16": os.path.join(_HERE, "libsentryfuse_f16.so")}
_libs = {}
_half = "bf16"

SF_F32, SF_BF16, SF_F16 = 0, 1, 2
SF_RELU, SF_GELU_ERF = 0, 1
SF_FLAG_FINAL_LN = 1

EXPORTS = ["sf_last_error", "sf_num_active", "sf_ffn_padded", "sf_gate_scores_to_masks",
           "sf_compact_heads_channels", "sf_sparse_gqa_workspace_bytes", "sf_sparse_gqa_forward",
           "sf_pruned_ffn_workspace_bytes", "sf_pruned_ffn_forward", "sf_encoder_workspace_bytes",
           "sf_encoder_forward", "sf_profile_begin", "sf_profile_end", "sf_compact_moe_experts",
           "sf_moe_ffn_workspace_bytes", "sf_moe_ffn_forward", "sf_gate_eval", "sf_budget_search",
           "sf_compact_heads_channels_fp8", "sf_ffn_fp8_padded", "sf_compact_ffn_fp8", "sf_quantize_fp8",
           "sf_pruned_ffn_fp8_workspace_bytes", "sf_pruned_ffn_fp8_forward", "sf_token_compact", "sf_token_scatter",
           "sf_encoder_forward_ragged", "sf_encoder_forward_fp8ffn", "sf_compact_heads_channels_f16",
           "sf_active_projection_rows", "sf_compact_proj_fp8", "sf_encoder_fp8_workspace_bytes",
           "sf_encoder_forward_fp8", "sf_proj_fp8_padded", "sf_presence_to_key_valid",
           "sf_sparse_gqa_static_capacity", "sf_sparse_gqa_forward_static", "sf_ceiling_mfma_launch",
           "sf_ceiling_copy_launch", "sf_token_pack_rows_max", "sf_token_pack", "sf_token_unpack",
           "sf_encoder_packed_workspace_bytes", "sf_encoder_forward_packed"]
SF_GATE_RELU, SF_GATE_TANH = 0, 1
SF_KERNEL_GEMM, SF_KERNEL_SCORE, SF_KERNEL_ATTEND = 0, 1, 2


class SfDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("B", C.c_int32), ("L", C.c_int32), ("d_model", C.c_int32),
                ("Hq", C.c_int32), ("Hk", C.c_int32), ("dh", C.c_int32), ("d_ff", C.c_int32),
                ("n_layers", C.c_int32), ("P", C.c_int32), ("dtype", C.c_int32), ("act", C.c_int32),
                ("c_factor", C.c_int32), ("U_override", C.c_int32), ("flags", C.c_uint32),
                ("ln_eps", C.c_float), ("ffn_pad", C.c_int32), ("n_sample", C.c_int32)]


class SfStrides(C.Structure):
    _fields_ = [("b", C.c_int64), ("h", C.c_int64), ("l", C.c_int64)]


_DENSE_FIELDS = ("Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo", "W1", "b1", "W2", "b2",
                 "ln1_g", "ln1_b", "ln2_g", "ln2_b")


class SfDenseLayer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _DENSE_FIELDS]


class SfCompactLayer(C.Structure):
    _fields_ = ([("k_head", C.c_int32), ("k_ffn", C.c_int32)]
                + [(n, C.c_void_p) for n in ("Wqkv", "bqkv", "WoT", "W1", "b1", "W2T", "bo", "b2",
                                             "ln1_g", "ln1_b", "ln2_g", "ln2_b", "head_group", "n_groups")])


_MOE_DENSE_FIELDS = ("Wr", "br", "W1", "b1", "W2", "b2", "ln_g", "ln_b")


class SfDenseLayerFp8(C.Structure):
    _fields_ = ([(n, C.c_void_p) for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2")]
                + [(n, C.c_float) for n in ("sq", "sk", "sv", "so", "s1", "s2")]
                + [(n, C.c_void_p) for n in ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")])


class SfFfnFp8(C.Structure):
    _fields_ = ([("k_ffn", C.c_int32), ("reserved", C.c_int32)]
                + [(n, C.c_void_p) for n in ("W1q", "b1", "W2Tq", "b2", "ln2_g", "ln2_b")]
                + [(n, C.c_float) for n in ("s1", "s2", "sx", "sh")])


class SfProjFp8(C.Structure):
    _fields_ = ([("k_head", C.c_int32), ("reserved", C.c_int32), ("Wqkv8", C.c_void_p), ("WoT8", C.c_void_p)]
                + [(n, C.c_float) for n in ("s_qkv", "so", "sx1", "sa")])


class SfTokenPackPlan(C.Structure):
    _fields_ = ([("Tc", C.c_int32)]
                + [(n, C.c_void_p) for n in ("len", "u_active", "row0", "ext", "valid_c", "blk_pattern", "src_row",
                                             "dst_row", "n_rows")])


class SfMoeDense(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _MOE_DENSE_FIELDS]


class SfMoeCompact(C.Structure):
    _fields_ = ([("n_experts", C.c_int32), ("top_k", C.c_int32), ("k_ffn_max", C.c_int32), ("reserved", C.c_int32)]
                + [(n, C.c_void_p) for n in ("Wr", "br", "W1", "b1", "W2T", "b2x", "ln_g", "ln_b", "k_ffn")])


class SfGateParams(C.Structure):
    _fields_ = ([("n_modalities", C.c_int32), ("hidden", C.c_int32), ("nonlin", C.c_int32), ("reserved", C.c_int32)]
                + [(n, C.c_void_p) for n in ("Wa", "ba", "Wb", "cb", "zeta", "gamma")])


class SentryFuseError(RuntimeError):
    pass


@contextlib.contextmanager
def use_half(half: str):
    """Within the block every call goes to the library build whose 16-bit type is `half` ("bf16" or "f16")."""
    global _half
    assert half in LIB_PATHS, half
    prev, _half = _half, half
    try:
        yield
    finally:
        _half = prev


def lib():
    """Load the HIP library (the build selected by use_half); never falls back to anything else."""
    if _half not in _libs:
        path = LIB_PATHS[_half]
        if not os.path.exists(path):
            raise SentryFuseError(f"{path} is missing: run `python -m paper_2604_08971_amd.build` first")
        L = C.CDLL(path)
        L.sf_last_error.restype = C.c_char_p
        for n in ("sf_sparse_gqa_workspace_bytes", "sf_pruned_ffn_workspace_bytes", "sf_encoder_workspace_bytes",
                  "sf_moe_ffn_workspace_bytes", "sf_pruned_ffn_fp8_workspace_bytes", "sf_encoder_fp8_workspace_bytes",
                  "sf_sparse_gqa_static_capacity", "sf_encoder_packed_workspace_bytes"):
            getattr(L, n).restype = C.c_size_t
        for n in ("sf_num_active", "sf_ffn_padded", "sf_gate_scores_to_masks", "sf_compact_heads_channels",
                  "sf_sparse_gqa_forward", "sf_pruned_ffn_forward", "sf_encoder_forward", "sf_profile_begin",
                  "sf_profile_end", "sf_compact_moe_experts", "sf_moe_ffn_forward", "sf_gate_eval",
                  "sf_budget_search", "sf_compact_heads_channels_fp8", "sf_ffn_fp8_padded", "sf_compact_ffn_fp8",
                  "sf_quantize_fp8", "sf_pruned_ffn_fp8_forward", "sf_token_compact", "sf_token_scatter",
                  "sf_encoder_forward_ragged", "sf_encoder_forward_fp8ffn", "sf_compact_heads_channels_f16",
                  "sf_active_projection_rows", "sf_compact_proj_fp8", "sf_encoder_forward_fp8", "sf_proj_fp8_padded",
                  "sf_presence_to_key_valid", "sf_sparse_gqa_forward_static", "sf_token_pack_rows_max",
                  "sf_token_pack", "sf_token_unpack", "sf_encoder_forward_packed"):
            getattr(L, n).restype = C.c_int32
        L.sf_token_pack_rows_max.argtypes = [C.POINTER(SfDesc)]
        L.sf_token_pack.argtypes = [C.POINTER(SfDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(SfTokenPackPlan),
                                    C.c_void_p, C.c_void_p]
        L.sf_token_unpack.argtypes = [C.POINTER(SfDesc), C.c_void_p, C.POINTER(SfTokenPackPlan), C.c_void_p, C.c_void_p]
        L.sf_encoder_packed_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer), C.c_int32]
        L.sf_encoder_forward_packed.argtypes = ([C.POINTER(SfDesc), C.POINTER(SfCompactLayer), C.c_void_p,
                                                 C.POINTER(SfTokenPackPlan)] + [C.c_void_p] * 8
                                                + [C.c_size_t, C.c_void_p])
        L.sf_sparse_gqa_forward.argtypes = [
            C.POINTER(SfDesc), C.c_int32, C.c_int32, C.c_void_p, SfStrides, C.c_void_p, SfStrides, C.c_void_p,
            SfStrides, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sf_sparse_gqa_forward_static.argtypes = L.sf_sparse_gqa_forward.argtypes[:19] + [C.c_void_p]
        L.sf_sparse_gqa_static_capacity.argtypes = []
        L.sf_ceiling_mfma_launch.restype = C.c_int64
        L.sf_ceiling_mfma_launch.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.sf_ceiling_copy_launch.restype = C.c_int32
        L.sf_ceiling_copy_launch.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sf_gate_scores_to_masks.argtypes = [C.POINTER(SfDesc)] + [C.c_void_p] * 12
        L.sf_presence_to_key_valid.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                               C.c_void_p]
        L.sf_compact_heads_channels.argtypes = [C.POINTER(SfDesc), C.c_int32, C.POINTER(SfDenseLayer),
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.POINTER(SfCompactLayer), C.c_void_p]
        L.sf_compact_heads_channels_f16.argtypes = [C.POINTER(SfDesc), C.c_int32, C.POINTER(SfDenseLayer)] + [
            C.c_void_p] * 4 + [C.POINTER(SfCompactLayer), C.c_void_p]
        L.sf_compact_heads_channels_fp8.argtypes = [C.POINTER(SfDesc), C.c_int32, C.POINTER(SfDenseLayerFp8),
                                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                    C.POINTER(SfCompactLayer), C.c_void_p]
        L.sf_pruned_ffn_forward.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer), C.c_void_p, C.c_void_p,
                                            C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sf_encoder_forward.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer), C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sf_encoder_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer)]
        L.sf_sparse_gqa_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.c_int32, C.c_int32]
        L.sf_pruned_ffn_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.c_int32]
        L.sf_pruned_ffn_fp8_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.c_int32]
        L.sf_encoder_forward_fp8ffn.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer), C.POINTER(SfFfnFp8)] + [
            C.c_void_p] * 13 + [C.c_size_t, C.c_void_p]
        L.sf_compact_proj_fp8.argtypes = [C.POINTER(SfDesc), C.c_int32, C.POINTER(SfDenseLayerFp8), C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.POINTER(SfProjFp8), C.c_void_p]
        L.sf_proj_fp8_padded.argtypes = [C.c_int32, C.c_int32]
        L.sf_encoder_fp8_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer)]
        L.sf_encoder_forward_fp8.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer), C.POINTER(SfFfnFp8),
                                             C.POINTER(SfProjFp8)] + [C.c_void_p] * 15 + [C.c_size_t, C.c_void_p]
        L.sf_token_compact.argtypes = [C.POINTER(SfDesc), C.c_void_p, C.c_void_p, C.c_int32] + [C.c_void_p] * 7
        L.sf_token_scatter.argtypes = [C.POINTER(SfDesc), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.sf_encoder_forward_ragged.argtypes = [C.POINTER(SfDesc), C.POINTER(SfCompactLayer)] + [C.c_void_p] * 11 + [
            C.c_size_t, C.c_void_p]
        L.sf_ffn_fp8_padded.argtypes = [C.c_int32]
        L.sf_compact_ffn_fp8.argtypes = [C.POINTER(SfDesc), C.c_int32, C.POINTER(SfDenseLayerFp8), C.c_void_p,
                                         C.POINTER(SfFfnFp8), C.c_void_p]
        L.sf_quantize_fp8.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_void_p, C.c_void_p]
        L.sf_pruned_ffn_fp8_forward.argtypes = [C.POINTER(SfDesc), C.POINTER(SfFfnFp8), C.c_void_p, C.c_void_p,
                                                C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_size_t, C.c_void_p]
        L.sf_compact_moe_experts.argtypes = [C.POINTER(SfDesc), C.POINTER(SfMoeDense), C.c_void_p, C.c_void_p,
                                             C.POINTER(SfMoeCompact), C.c_void_p]
        L.sf_moe_ffn_workspace_bytes.argtypes = [C.POINTER(SfDesc), C.POINTER(SfMoeCompact)]
        L.sf_moe_ffn_forward.argtypes = [C.POINTER(SfDesc), C.POINTER(SfMoeCompact), C.c_void_p, C.c_void_p, C.c_int32,
                                         C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
        L.sf_gate_eval.argtypes = [C.POINTER(SfDesc), C.POINTER(SfGateParams), C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p]
        L.sf_budget_search.argtypes = [C.POINTER(SfDesc), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
        L.sf_profile_begin.argtypes = [C.c_int32, C.c_int32]
        L.sf_profile_end.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.sf_num_active.argtypes = [C.POINTER(SfDesc)]
        L.sf_active_projection_rows.argtypes = [C.POINTER(SfDesc), C.c_int32]
        L.sf_ffn_padded.argtypes = [C.POINTER(SfDesc), C.c_int32]
        _libs[_half] = L
    return _libs[_half]


def _check(rc: int, what: str):
    if rc != 0:
        raise SentryFuseError(f"{what} failed with status {rc}: {lib().sf_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == SF_BF16 else torch.float16 if dtype == SF_F16 else torch.float32


def make_desc(B, L, d_model, Hq, Hk, dh, d_ff, n_layers=1, P=1, dtype=SF_BF16, act=SF_RELU, c_factor=5,
              U_override=-1, final_ln=False, ln_eps=1e-5, ffn_pad=64, n_sample=0) -> SfDesc:
    return SfDesc(C.sizeof(SfDesc), B, L, d_model, Hq, Hk, dh, d_ff, n_layers, P, dtype, act, c_factor,
                  U_override, SF_FLAG_FINAL_LN if final_ln else 0, ln_eps, ffn_pad, n_sample)


def num_active(desc: SfDesc) -> int:
    u = lib().sf_num_active(C.byref(desc))
    if u < 0:
        _check(u, "sf_num_active")
    return int(u)


def active_projection_rows(desc: SfDesc, k_head: int) -> int:
    r = lib().sf_active_projection_rows(C.byref(desc), int(k_head))
    if r < 0:
        _check(r, "sf_active_projection_rows")
    return int(r)


def ffn_padded(desc: SfDesc, k_ffn: int) -> int:
    r = lib().sf_ffn_padded(C.byref(desc), int(k_ffn))
    if r < 0:
        _check(r, "sf_ffn_padded")
    return int(r)


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


_prof_cap = 0


def ceiling_mfma_launch(workgroups: int, iters: int, random_operands: bool, sink: torch.Tensor) -> int:
    """One launch of the register-only MFMA loop; returns its flops."""
    assert sink.dtype == torch.float32 and sink.numel() >= workgroups
    fl = lib().sf_ceiling_mfma_launch(int(workgroups), int(iters), int(random_operands), _ptr(sink), _stream())
    if fl < 0:
        _check(int(fl), "sf_ceiling_mfma_launch")
    return int(fl)


def ceiling_copy_launch(src: torch.Tensor, dst: torch.Tensor):
    assert src.is_contiguous() and dst.is_contiguous() and src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _check(lib().sf_ceiling_copy_launch(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()),
           "sf_ceiling_copy_launch")


def profile_begin(kernel_class: int, max_launches: int):
    global _prof_cap
    _check(lib().sf_profile_begin(kernel_class, max_launches), "sf_profile_begin")
    _prof_cap = max_launches


def profile_end(each: bool = False):
    """Returns (number of launches timed, sum of their durations in ms[, list of durations in launch order])."""
    n, ms = C.c_int32(0), C.c_float(0.0)
    buf = (C.c_float * max(_prof_cap, 1))() if each else None
    _check(lib().sf_profile_end(C.byref(n), C.byref(ms), buf), "sf_profile_end")
    if each:
        return int(n.value), float(ms.value), [float(buf[i]) for i in range(int(n.value))]
    return int(n.value), float(ms.value)


# ------------------------------------------------------- SentryGate: Eq. (1) and the global threshold
def gate_eval(desc: SfDesc, gate: Dict[str, torch.Tensor], pattern_bits: torch.Tensor, nonlin: int = SF_GATE_RELU):
    """gate: Wa [nl,Hd,M], ba [nl,Hd] | None, Wb [nl,Hq+F,Hd], cb [nl,Hq+F] | None, zeta [nl,Hq+F], gamma [nl] (fp32,
    contiguous); pattern_bits [P] int32.  Returns (g_head [nl,P,Hq], g_ffn [nl,P,F]) fp32."""
    nl, P, Hq, F = desc.n_layers, desc.P, desc.Hq, desc.d_ff
    Wa, Wb = gate["Wa"], gate["Wb"]
    Hd, M = Wa.shape[1], Wa.shape[2]
    for k, shape in (("Wa", (nl, Hd, M)), ("ba", (nl, Hd)), ("Wb", (nl, Hq + F, Hd)), ("cb", (nl, Hq + F)),
                     ("zeta", (nl, Hq + F)), ("gamma", (nl,))):
        t = gate.get(k)
        assert t is None or (t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape), k
    assert pattern_bits.dtype == torch.int32 and tuple(pattern_bits.shape) == (P,)
    gp = SfGateParams(M, Hd, nonlin, 0, *[_ptr(gate.get(k)) for k in ("Wa", "ba", "Wb", "cb", "zeta", "gamma")])
    g_head = torch.empty((nl, P, Hq), dtype=torch.float32, device=Wa.device)
    g_ffn = torch.empty((nl, P, F), dtype=torch.float32, device=Wa.device)
    _check(lib().sf_gate_eval(C.byref(desc), C.byref(gp), _ptr(pattern_bits), _ptr(g_head), _ptr(g_ffn), _stream()),
           "sf_gate_eval")
    return g_head, g_ffn


def budget_search(desc: SfDesc, g_head: torch.Tensor, g_ffn: torch.Tensor, pattern: int, c_head: Sequence[int],
                  c_group: Sequence[int], c_ffn: Sequence[int], c_fixed: int, budget: int):
    """Returns device tensors: dict(tau [1] f32, k_head [nl] i32, k_ffn [nl] i32, cost [1] i64, feasible [1] i32)."""
    nl = desc.n_layers
    assert g_head.dtype == torch.float32 and g_head.is_contiguous() and tuple(g_head.shape) == (nl, desc.P, desc.Hq)
    assert g_ffn.dtype == torch.float32 and g_ffn.is_contiguous() and tuple(g_ffn.shape) == (nl, desc.P, desc.d_ff)
    assert len(c_head) == nl and len(c_group) == nl and len(c_ffn) == nl
    dev = g_head.device
    out = {"tau": torch.empty(1, dtype=torch.float32, device=dev), "k_head": torch.empty(nl, dtype=torch.int32, device=dev),
           "k_ffn": torch.empty(nl, dtype=torch.int32, device=dev), "cost": torch.empty(1, dtype=torch.int64, device=dev),
           "feasible": torch.empty(1, dtype=torch.int32, device=dev)}
    ch, cg, cf = ((C.c_int64 * nl)(*[int(v) for v in a]) for a in (c_head, c_group, c_ffn))
    _check(lib().sf_budget_search(C.byref(desc), _ptr(g_head), _ptr(g_ffn), int(pattern), C.cast(ch, C.c_void_p),
                                  C.cast(cg, C.c_void_p), C.cast(cf, C.c_void_p), int(c_fixed), int(budget),
                                  _ptr(out["tau"]), _ptr(out["k_head"]), _ptr(out["k_ffn"]), _ptr(out["cost"]),
                                  _ptr(out["feasible"]), _stream()), "sf_budget_search")
    return out


# ------------------------------------------------------------- presence mask -> allowed keys
def presence_to_key_valid(presence: torch.Tensor, tok_modality: torch.Tensor,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """key_valid [B, L] u8 from the presence masks [B, M] u8 and the token -> modality map [L] int32 (-1: no modality)."""
    assert presence.dtype == torch.uint8 and presence.is_contiguous() and presence.dim() == 2
    assert tok_modality.dtype == torch.int32 and tok_modality.is_contiguous() and tok_modality.dim() == 1
    B, M = presence.shape
    L = tok_modality.shape[0]
    if out is None:
        out = torch.empty((B, L), dtype=torch.uint8, device=presence.device)
    assert out.dtype == torch.uint8 and out.is_contiguous() and tuple(out.shape) == (B, L)
    _check(lib().sf_presence_to_key_valid(_ptr(presence), _ptr(tok_modality), B, M, L, _ptr(out), _stream()),
           "sf_presence_to_key_valid")
    return out


# --------------------------------------------------------------------------- a1
def gate_scores_to_masks(desc: SfDesc, g_head: torch.Tensor, g_ffn: torch.Tensor, k_head: Sequence[int],
                         k_ffn: Sequence[int], out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    nl, P, Hq, Hk, F = desc.n_layers, desc.P, desc.Hq, desc.Hk, desc.d_ff
    dev = g_head.device
    assert g_head.dtype == torch.float32 and g_ffn.dtype == torch.float32
    assert tuple(g_head.shape) == (nl, P, Hq) and tuple(g_ffn.shape) == (nl, P, F)
    assert g_head.is_contiguous() and g_ffn.is_contiguous()
    out = out if out is not None else {
        "head_mask": torch.empty((nl, P, Hq), dtype=torch.uint8, device=dev),
        "ffn_mask": torch.empty((nl, P, F), dtype=torch.uint8, device=dev),
        "head_idx": torch.empty((nl, P, Hq), dtype=torch.int32, device=dev),
        "ffn_idx": torch.empty((nl, P, F), dtype=torch.int32, device=dev),
        "group_idx": torch.empty((nl, P, Hk), dtype=torch.int32, device=dev),
        "n_groups": torch.empty((nl, P), dtype=torch.int32, device=dev),
        "head_group": torch.empty((nl, P, Hq), dtype=torch.int32, device=dev),
    }
    kh = (C.c_int32 * nl)(*[int(k) for k in k_head])
    kf = (C.c_int32 * nl)(*[int(k) for k in k_ffn])
    rc = lib().sf_gate_scores_to_masks(
        C.byref(desc), _ptr(g_head), _ptr(g_ffn), C.cast(kh, C.c_void_p), C.cast(kf, C.c_void_p),
        _ptr(out["head_mask"]), _ptr(out["ffn_mask"]), _ptr(out["head_idx"]), _ptr(out["ffn_idx"]),
        _ptr(out["group_idx"]), _ptr(out["n_groups"]), _ptr(out["head_group"]), _stream())
    _check(rc, "sf_gate_scores_to_masks")
    return out


# --------------------------------------------------------------------------- a2
class CompactLayer:
    """Device buffers of one compacted layer (all P patterns) plus the C struct."""

    def __init__(self, desc: SfDesc, dense: Dict[str, torch.Tensor], k_head: int, k_ffn: int,
                 head_group: torch.Tensor, n_groups: torch.Tensor):
        P, dh, d, Hk = desc.P, desc.dh, desc.d_model, desc.Hk
        dt, dev = torch_dtype(desc.dtype), dense["Wq"].device
        self.k_head, self.k_ffn = int(k_head), int(k_ffn)
        self.Fp = ffn_padded(desc, k_ffn)
        self.Nqkv = (self.k_head + 2 * Hk) * dh
        e = lambda *s: torch.empty(s, dtype=dt, device=dev)
        self.Wqkv = e(P, self.Nqkv, d)
        self.bqkv = e(P, self.Nqkv) if dense.get("bq") is not None else None
        self.WoT = e(P, d, self.k_head * dh)
        self.W1 = e(P, self.Fp, d)
        self.b1 = e(P, self.Fp) if dense.get("b1") is not None else None
        self.W2T = e(P, d, self.Fp)
        self.dense = dense                     # keeps bo, b2, ln* alive
        self.head_group, self.n_groups = head_group, n_groups
        s = SfCompactLayer()
        s.k_head, s.k_ffn = self.k_head, self.k_ffn
        for n in ("Wqkv", "bqkv", "WoT", "W1", "b1", "W2T"):
            t = getattr(self, n)
            setattr(s, n, None if t is None else t.data_ptr())
        for n in ("bo", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b"):
            t = dense.get(n)
            setattr(s, n, None if t is None else t.data_ptr())
        s.head_group = head_group.data_ptr()
        s.n_groups = n_groups.data_ptr()
        self.struct = s


def dense_struct(dense: Dict[str, torch.Tensor]) -> SfDenseLayer:
    s = SfDenseLayer()
    for n in _DENSE_FIELDS:
        t = dense.get(n)
        if t is not None:
            assert t.is_contiguous()
        setattr(s, n, None if t is None else t.data_ptr())
    return s


def compact_heads_channels(desc: SfDesc, layer: int, dense: Dict[str, torch.Tensor],
                           masks: Dict[str, torch.Tensor], k_head: int, k_ffn: int,
                           out: Optional[CompactLayer] = None) -> CompactLayer:
    """Fills the compact buffers of `layer` on the GPU (allocating them unless `out`,
    built for the same masks tensors and counts, is given)."""
    if out is None:
        hg = masks["head_group"][layer]
        ng = masks["n_groups"][layer]
        cl = CompactLayer(desc, dense, k_head, k_ffn, hg, ng)
    else:
        cl = out
        assert cl.k_head == int(k_head) and cl.k_ffn == int(k_ffn)
        assert cl.head_group.data_ptr() == masks["head_group"][layer].data_ptr()
    ds = dense_struct(dense)
    rc = lib().sf_compact_heads_channels(C.byref(desc), int(layer), C.byref(ds), _ptr(masks["head_idx"]),
                                         _ptr(masks["group_idx"]), _ptr(masks["n_groups"]),
                                         _ptr(masks["ffn_idx"]), C.byref(cl.struct), _stream())
    _check(rc, "sf_compact_heads_channels")
    return cl


# ------------------------------------------------------------------------ a4-a7
def compact_heads_channels_fp8(desc: SfDesc, layer: int, dense8: Dict[str, torch.Tensor], scales: Dict[str, float],
                               masks: Dict[str, torch.Tensor], k_head: int, k_ffn: int,
                               out: Optional[CompactLayer] = None) -> CompactLayer:
    """dense8: Wq, Wk, Wv, Wo, W1, W2 as uint8 (OCP E4M3 codes, shapes of the dense layer) plus the biases and
    LayerNorm vectors in the model dtype; scales: one float per weight matrix, keyed like the matrices."""
    for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2"):
        assert dense8[n].dtype == torch.uint8 and dense8[n].is_contiguous(), n
    cl = out if out is not None else CompactLayer(desc, dense8, k_head, k_ffn, masks["head_group"][layer],
                                                  masks["n_groups"][layer])
    ds = SfDenseLayerFp8(*[_ptr(dense8[n]) for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2")],
                         *[float(scales[n]) for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2")],
                         *[_ptr(dense8.get(n)) for n in ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")])
    rc = lib().sf_compact_heads_channels_fp8(C.byref(desc), layer, C.byref(ds), _ptr(masks["head_idx"]),
                                             _ptr(masks["group_idx"]), _ptr(masks["n_groups"]), _ptr(masks["ffn_idx"]),
                                             C.byref(cl.struct), _stream())
    _check(rc, "sf_compact_heads_channels_fp8")
    return cl


def compact_heads_channels_f16(desc: SfDesc, layer: int, dense16: Dict[str, torch.Tensor],
                               masks: Dict[str, torch.Tensor], k_head: int, k_ffn: int,
                               out: Optional[CompactLayer] = None) -> CompactLayer:
    """dense16: Wq, Wk, Wv, Wo, W1, W2 as torch.float16 (shapes of the dense layer), biases and LayerNorm vectors in
    the model dtype."""
    for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2"):
        assert dense16[n].dtype == torch.float16 and dense16[n].is_contiguous(), n
    cl = out if out is not None else CompactLayer(desc, dense16, k_head, k_ffn, masks["head_group"][layer],
                                                  masks["n_groups"][layer])
    ds = SfDenseLayer(*[_ptr(dense16.get(n)) for n in _DENSE_FIELDS])
    rc = lib().sf_compact_heads_channels_f16(C.byref(desc), layer, C.byref(ds), _ptr(masks["head_idx"]),
                                             _ptr(masks["group_idx"]), _ptr(masks["n_groups"]), _ptr(masks["ffn_idx"]),
                                             C.byref(cl.struct), _stream())
    _check(rc, "sf_compact_heads_channels_f16")
    return cl


def _strides4(t: torch.Tensor) -> SfStrides:
    assert t.dim() == 4 and t.stride(3) == 1
    return SfStrides(t.stride(0), t.stride(1), t.stride(2))


def sparse_gqa_workspace_bytes(desc: SfDesc, nH: int, nG: int) -> int:
    return int(lib().sf_sparse_gqa_workspace_bytes(C.byref(desc), nH, nG))


def sparse_gqa_forward(desc: SfDesc, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                       head_group: torch.Tensor, pattern_id: Optional[torch.Tensor] = None,
                       key_valid: Optional[torch.Tensor] = None, forced_sel: Optional[torch.Tensor] = None,
                       v_transposed: bool = False, want_sel: bool = True, want_score: bool = False,
                       ws: Optional[torch.Tensor] = None, sample_idx: Optional[torch.Tensor] = None):
    """Q [B,nH,L,dh], K [B,nG,L,dh], V [B,nG,L,dh] (or [B,nG,dh,L] with v_transposed);
    last dimension contiguous.  sample_idx [B, desc.n_sample] int32: key sample of the sparsity score.
    Returns (O [B,L,nH*dh], sel [B,nH,U] | None, score [B,nH,L] | None)."""
    _check_sample(desc, sample_idx, Q.shape[0])
    B, nH, L, dh = Q.shape
    nG = K.shape[1]
    U = num_active(desc)
    dev = Q.device
    O = torch.empty((B, L, nH * dh), dtype=Q.dtype, device=dev)
    sel = torch.empty((B, nH, max(U, 1)), dtype=torch.int32, device=dev) if want_sel else None
    score = torch.full((B, nH, L), float("nan"), dtype=torch.float32, device=dev) if want_score else None
    if ws is None:
        ws = workspace(sparse_gqa_workspace_bytes(desc, nH, nG), dev)
    rc = lib().sf_sparse_gqa_forward(
        C.byref(desc), nH, nG, _ptr(Q), _strides4(Q), _ptr(K), _strides4(K), _ptr(V), _strides4(V),
        int(v_transposed), _ptr(head_group), _ptr(pattern_id), _ptr(key_valid), _ptr(sample_idx),
        _ptr(forced_sel), _ptr(O),
        nH * dh, _ptr(sel), _ptr(score), _ptr(ws), ws.numel(), _stream())
    _check(rc, "sf_sparse_gqa_forward")
    if sel is not None:
        sel = sel[:, :, :U]
    return O, sel, score


def sparse_gqa_static_capacity() -> int:
    return int(lib().sf_sparse_gqa_static_capacity())


def sparse_gqa_forward_static(desc: SfDesc, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                              head_group: torch.Tensor, O: torch.Tensor, pattern_id: Optional[torch.Tensor] = None,
                              key_valid: Optional[torch.Tensor] = None, forced_sel: Optional[torch.Tensor] = None,
                              v_transposed: bool = False, sel: Optional[torch.Tensor] = None,
                              score: Optional[torch.Tensor] = None, sample_idx: Optional[torch.Tensor] = None):
    """sf_sparse_gqa_forward_static: every buffer (O [B,L,nH*dh], optionally sel [B,nH,U] and score [B,nH,L]) is the
    caller's, the scratch memory is the library's built-in buffer; nothing is allocated by this call."""
    _check_sample(desc, sample_idx, Q.shape[0])
    B, nH, L, dh = Q.shape
    nG = K.shape[1]
    assert O.is_contiguous() and tuple(O.shape) == (B, L, nH * dh) and O.dtype == Q.dtype
    rc = lib().sf_sparse_gqa_forward_static(
        C.byref(desc), nH, nG, _ptr(Q), _strides4(Q), _ptr(K), _strides4(K), _ptr(V), _strides4(V),
        int(v_transposed), _ptr(head_group), _ptr(pattern_id), _ptr(key_valid), _ptr(sample_idx),
        _ptr(forced_sel), _ptr(O), nH * dh, _ptr(sel), _ptr(score), _stream())
    _check(rc, "sf_sparse_gqa_forward_static")


def _check_sample(desc: SfDesc, sample_idx: Optional[torch.Tensor], B: int):
    if sample_idx is not None:
        assert sample_idx.dtype == torch.int32 and sample_idx.is_contiguous()
        assert tuple(sample_idx.shape) == (B, desc.n_sample), (tuple(sample_idx.shape), (B, desc.n_sample))


# --------------------------------------------------------------------------- a9
def pruned_ffn_forward(desc: SfDesc, layer: CompactLayer, X: torch.Tensor,
                       pattern_id: Optional[torch.Tensor] = None, pre_ln: bool = True,
                       add_residual: bool = True, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    assert X.is_contiguous()
    Y = torch.empty_like(X)
    if ws is None:
        ws = workspace(lib().sf_pruned_ffn_workspace_bytes(C.byref(desc), layer.k_ffn), X.device)
    rc = lib().sf_pruned_ffn_forward(C.byref(desc), C.byref(layer.struct), _ptr(X), _ptr(pattern_id),
                                     int(pre_ln), int(add_residual), _ptr(Y), _ptr(ws), ws.numel(), _stream())
    _check(rc, "sf_pruned_ffn_forward")
    return Y


# ---------------------------------------------------------- pruned FFN in FP8 arithmetic
class CompactFfnFp8:
    """FFN weights of one layer as E4M3 codes, compacted for all patterns: owns the padded device buffers."""

    def __init__(self, desc: SfDesc, dense8: Dict[str, torch.Tensor], scales: Dict[str, float], k_ffn: int,
                 sx: float, sh: float):
        P, d = desc.P, desc.d_model
        dev = dense8["W1"].device
        self.k_ffn = int(k_ffn)
        self.Fp8 = int(lib().sf_ffn_fp8_padded(self.k_ffn))
        self.dense8 = dense8
        self.W1q = torch.empty((P, self.Fp8, d), dtype=torch.uint8, device=dev)
        self.W2Tq = torch.empty((P, d, self.Fp8), dtype=torch.uint8, device=dev)
        self.b1 = (torch.empty((P, self.Fp8), dtype=dense8["b1"].dtype, device=dev)
                   if dense8.get("b1") is not None else None)
        self.struct = SfFfnFp8(self.k_ffn, 0, _ptr(self.W1q), _ptr(self.b1), _ptr(self.W2Tq), _ptr(dense8.get("b2")),
                               _ptr(dense8.get("ln2_g")), _ptr(dense8.get("ln2_b")), float(scales["W1"]),
                               float(scales["W2"]), float(sx), float(sh))


def compact_ffn_fp8(desc: SfDesc, layer: int, dense8: Dict[str, torch.Tensor], scales: Dict[str, float],
                    masks: Dict[str, torch.Tensor], k_ffn: int, sx: float, sh: float) -> CompactFfnFp8:
    """dense8: W1, W2 [d_ff, d] uint8 (E4M3 codes), b1, b2, ln2_g, ln2_b in bf16; scales: W1, W2."""
    for n in ("W1", "W2"):
        assert dense8[n].dtype == torch.uint8 and dense8[n].is_contiguous(), n
    cf = CompactFfnFp8(desc, dense8, scales, k_ffn, sx, sh)
    nul = C.c_void_p(None)
    ds = SfDenseLayerFp8(nul, nul, nul, nul, _ptr(dense8["W1"]), _ptr(dense8["W2"]), 0.0, 0.0, 0.0, 0.0,
                         float(scales["W1"]), float(scales["W2"]), nul, nul, nul, nul, _ptr(dense8.get("b1")),
                         _ptr(dense8.get("b2")), nul, nul, _ptr(dense8.get("ln2_g")), _ptr(dense8.get("ln2_b")))
    rc = lib().sf_compact_ffn_fp8(C.byref(desc), layer, C.byref(ds), _ptr(masks["ffn_idx"]), C.byref(cf.struct),
                                  _stream())
    _check(rc, "sf_compact_ffn_fp8")
    return cf


def quantize_fp8(x: torch.Tensor, scale: float) -> torch.Tensor:
    """E4M3 codes of x / scale (x fp32 or bf16, contiguous)."""
    assert x.is_contiguous() and x.dtype in (torch.float32, torch.bfloat16)
    codes = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    rc = lib().sf_quantize_fp8(_ptr(x), SF_F32 if x.dtype == torch.float32 else SF_BF16, x.numel(), float(scale),
                               _ptr(codes), _stream())
    _check(rc, "sf_quantize_fp8")
    return codes


def pruned_ffn_fp8_forward(desc: SfDesc, ffn: CompactFfnFp8, X: torch.Tensor,
                           pattern_id: Optional[torch.Tensor] = None, pre_ln: bool = True,
                           add_residual: bool = True, want_codes: bool = False, ws: Optional[torch.Tensor] = None):
    """X [B, L, d] bf16.  Returns Y, or (Y, xq [B*L, d], hq [B*L, Fp8]) with want_codes."""
    assert X.is_contiguous() and X.dtype == torch.bfloat16
    Y = torch.empty_like(X)
    rows = X.numel() // X.shape[-1]
    xq = torch.empty((rows, X.shape[-1]), dtype=torch.uint8, device=X.device) if want_codes else None
    hq = torch.empty((rows, ffn.Fp8), dtype=torch.uint8, device=X.device) if want_codes else None
    if ws is None:
        ws = workspace(lib().sf_pruned_ffn_fp8_workspace_bytes(C.byref(desc), ffn.k_ffn), X.device)
    rc = lib().sf_pruned_ffn_fp8_forward(C.byref(desc), C.byref(ffn.struct), _ptr(X), _ptr(pattern_id), int(pre_ln),
                                         int(add_residual), _ptr(Y), _ptr(xq), _ptr(hq), _ptr(ws), ws.numel(),
                                         _stream())
    _check(rc, "sf_pruned_ffn_fp8_forward")
    return (Y, xq, hq) if want_codes else Y


# ---------------------------------------------------------- Sparse-MoE FFN with pruned experts
class CompactMoe:
    """Compacted experts of one MoE block: owns the padded device buffers."""

    def __init__(self, desc: SfDesc, dense: Dict[str, torch.Tensor], top_k: int, k_ffn: Sequence[int]):
        E, F, d = dense["W1"].shape
        assert F == desc.d_ff and d == desc.d_model and len(k_ffn) == E
        P = desc.P
        dt, dev = dense["W1"].dtype, dense["W1"].device
        self.k_ffn = [int(k) for k in k_ffn]
        self.E, self.top_k = E, int(top_k)
        self.Fp = ffn_padded(desc, max(self.k_ffn))
        self.dense = dense
        self.W1 = torch.empty((P, E, self.Fp, d), dtype=dt, device=dev)
        self.b1 = torch.empty((P, E, self.Fp), dtype=dt, device=dev) if dense.get("b1") is not None else None
        self.W2T = torch.empty((P, E, d, self.Fp), dtype=dt, device=dev)
        self.b2x = torch.empty((P, E, d), dtype=dt, device=dev) if dense.get("b2") is not None else None
        self.k_ffn_dev = torch.zeros(E, dtype=torch.int32, device=dev)
        self.struct = SfMoeCompact(E, self.top_k, max(self.k_ffn), 0, _ptr(dense["Wr"]), _ptr(dense.get("br")),
                                   _ptr(self.W1), _ptr(self.b1), _ptr(self.W2T), _ptr(self.b2x),
                                   _ptr(dense.get("ln_g")), _ptr(dense.get("ln_b")), _ptr(self.k_ffn_dev))


def compact_moe_experts(desc: SfDesc, dense: Dict[str, torch.Tensor], ffn_idx: torch.Tensor, top_k: int,
                        k_ffn: Sequence[int], out: Optional[CompactMoe] = None) -> CompactMoe:
    """dense: Wr [E,d], br [E] | None, W1 [E,F,d], b1 [E,F] | None, W2 [E,F,d], b2 [E,d] | None, ln_g, ln_b [d];
    ffn_idx [E,P,F] int32 kept channels (ascending) of every expert and pattern."""
    cm = out if out is not None else CompactMoe(desc, dense, top_k, k_ffn)
    E = cm.E
    assert ffn_idx.dtype == torch.int32 and ffn_idx.is_contiguous() and tuple(ffn_idx.shape) == (E, desc.P, desc.d_ff)
    ds = SfMoeDense(*[_ptr(dense.get(n)) for n in _MOE_DENSE_FIELDS])
    kf = (C.c_int32 * E)(*cm.k_ffn)
    _check(lib().sf_compact_moe_experts(C.byref(desc), C.byref(ds), _ptr(ffn_idx), C.cast(kf, C.c_void_p),
                                        C.byref(cm.struct), _stream()), "sf_compact_moe_experts")
    return cm


def moe_ffn_workspace_bytes(desc: SfDesc, moe: CompactMoe) -> int:
    return int(lib().sf_moe_ffn_workspace_bytes(C.byref(desc), C.byref(moe.struct)))


def moe_ffn_forward(desc: SfDesc, moe: CompactMoe, X: torch.Tensor, pattern_id: Optional[torch.Tensor] = None,
                    pre_ln: bool = True, add_residual: bool = True, forced_route: Optional[torch.Tensor] = None,
                    want_route: bool = False, out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """X [B*L, d].  Returns Y, or (Y, route [B*L,k] int32, weight [B*L,k] f32, logit [B*L,E] f32) with want_route."""
    assert X.is_contiguous()
    rows = X.shape[0]
    Y = torch.empty_like(X) if out is None else out
    route = weight = logit = None
    if want_route:
        route = torch.empty((rows, moe.top_k), dtype=torch.int32, device=X.device)
        weight = torch.empty((rows, moe.top_k), dtype=torch.float32, device=X.device)
        logit = torch.empty((rows, moe.E), dtype=torch.float32, device=X.device)
    if forced_route is not None:
        assert forced_route.dtype == torch.int32 and forced_route.is_contiguous()
        assert tuple(forced_route.shape) == (rows, moe.top_k)
    if ws is None:
        ws = workspace(moe_ffn_workspace_bytes(desc, moe), X.device)
    rc = lib().sf_moe_ffn_forward(C.byref(desc), C.byref(moe.struct), _ptr(X), _ptr(pattern_id), int(pre_ln),
                                  int(add_residual), _ptr(forced_route), _ptr(Y), _ptr(route), _ptr(weight),
                                  _ptr(logit), _ptr(ws), ws.numel(), _stream())
    _check(rc, "sf_moe_ffn_forward")
    return (Y, route, weight, logit) if want_route else Y


# -------------------------------------------------------------------------- a10
def layer_array(layers: List[CompactLayer]):
    arr = (SfCompactLayer * len(layers))()
    for i, l in enumerate(layers):
        arr[i] = l.struct
    return arr


def encoder_workspace_bytes(desc: SfDesc, layers: List[CompactLayer]) -> int:
    return int(lib().sf_encoder_workspace_bytes(C.byref(desc), layer_array(layers)))


def encoder_forward(desc: SfDesc, layers: List[CompactLayer], X: torch.Tensor,
                    pattern_id: Optional[torch.Tensor] = None, key_valid: Optional[torch.Tensor] = None,
                    final_ln: Optional[Dict[str, torch.Tensor]] = None,
                    forced_sel: Optional[torch.Tensor] = None, want_sel: bool = False,
                    want_score: bool = False, out: Optional[torch.Tensor] = None,
                    ws: Optional[torch.Tensor] = None, sample_idx: Optional[torch.Tensor] = None):
    """sample_idx [B, desc.n_sample] int32: key sample of the sparsity score (every layer).
    Returns (Y [B,L,d], sel [nl,B,Hq'max,U] | None, score [nl,B,Hq'max,L] | None)."""
    assert X.is_contiguous()
    _check_sample(desc, sample_idx, X.shape[0])
    B, L, _ = X.shape
    nl = desc.n_layers
    U = num_active(desc)
    khmax = max(l.k_head for l in layers)
    dev = X.device
    Y = torch.empty_like(X) if out is None else out
    sel = torch.full((nl, B, khmax, max(U, 1)), -1, dtype=torch.int32, device=dev) if want_sel else None
    score = torch.full((nl, B, khmax, L), float("-inf"), dtype=torch.float32, device=dev) if want_score else None
    if sel is not None and U == 0:
        sel = sel[..., :0].contiguous()
    arr = layer_array(layers)
    if ws is None:
        ws = workspace(lib().sf_encoder_workspace_bytes(C.byref(desc), arr), dev)
    fg = None if final_ln is None else final_ln["g"]
    fb = None if final_ln is None else final_ln["b"]
    rc = lib().sf_encoder_forward(C.byref(desc), arr, _ptr(X), _ptr(pattern_id), _ptr(key_valid),
                                  _ptr(sample_idx), _ptr(fg), _ptr(fb), _ptr(forced_sel), _ptr(Y), _ptr(sel if U > 0 else None),
                                  _ptr(score), _ptr(ws), ws.numel(), _stream())
    _check(rc, "sf_encoder_forward")
    return Y, sel, score


# ---------------------------------------------------------- token compaction (absent modalities contribute no tokens)
def token_compact(desc: SfDesc, X: torch.Tensor, token_valid: torch.Tensor, Lc: int) -> Dict[str, torch.Tensor]:
    """X [B,L,d], token_valid [B,L] uint8.  Returns Xc [B,Lc,d], valid_c [B,Lc] u8, row_index [B,Lc], slot_of [B,L],
    len [B], u_active [B] (int32)."""
    assert X.is_contiguous() and token_valid.is_contiguous() and token_valid.dtype == torch.uint8
    B, L, d = X.shape
    dev = X.device
    i32 = lambda *sh: torch.empty(sh, dtype=torch.int32, device=dev)
    out = dict(Xc=torch.empty((B, Lc, d), dtype=X.dtype, device=dev),
               valid_c=torch.empty((B, Lc), dtype=torch.uint8, device=dev), row_index=i32(B, Lc), slot_of=i32(B, L),
               len=i32(B), u_active=i32(B))
    rc = lib().sf_token_compact(C.byref(desc), _ptr(X), _ptr(token_valid), int(Lc), _ptr(out["Xc"]), _ptr(out["valid_c"]),
                                _ptr(out["row_index"]), _ptr(out["slot_of"]), _ptr(out["len"]), _ptr(out["u_active"]),
                                _stream())
    _check(rc, "sf_token_compact")
    return out


def token_scatter(desc: SfDesc, Yc: torch.Tensor, slot_of: torch.Tensor) -> torch.Tensor:
    """Yc [B,Lc,d] -> Y [B,L,d] (desc of the full sequence), zero rows for dropped tokens."""
    assert Yc.is_contiguous()
    B, Lc, d = Yc.shape
    Y = torch.empty((B, desc.L, d), dtype=Yc.dtype, device=Yc.device)
    _check(lib().sf_token_scatter(C.byref(desc), _ptr(Yc), _ptr(slot_of), int(Lc), _ptr(Y), _stream()), "sf_token_scatter")
    return Y


class TokenPackPlan:
    """The device arrays of a packed token layout (sf_token_pack_plan) and the struct that points at them."""

    def __init__(self, B: int, L: int, Tc: int, device):
        i32 = lambda *sh: torch.empty(sh, dtype=torch.int32, device=device)
        self.B, self.L, self.Tc = B, L, Tc
        self.len, self.u_active, self.row0, self.ext = i32(B), i32(B), i32(B), i32(B)
        self.valid_c = torch.empty((B, L), dtype=torch.uint8, device=device)
        self.blk_pattern, self.src_row, self.dst_row, self.n_rows = i32(Tc // 256), i32(Tc), i32(B, L), i32(2)
        self.c = SfTokenPackPlan()
        self.c.Tc = Tc
        for n in ("len", "u_active", "row0", "ext", "valid_c", "blk_pattern", "src_row", "dst_row", "n_rows"):
            setattr(self.c, n, getattr(self, n).data_ptr())


def token_pack_rows_max(desc: SfDesc) -> int:
    n = lib().sf_token_pack_rows_max(C.byref(desc))
    _check(min(n, 0), "sf_token_pack_rows_max")
    return int(n)


def encoder_packed_workspace_bytes(desc: SfDesc, layers: List[CompactLayer], Tc: int) -> int:
    return int(lib().sf_encoder_packed_workspace_bytes(C.byref(desc), layer_array(layers), int(Tc)))


def token_pack(desc: SfDesc, X: torch.Tensor, token_valid: torch.Tensor, pattern_id: Optional[torch.Tensor],
               Tc: Optional[int] = None, plan: Optional[TokenPackPlan] = None, out: Optional[torch.Tensor] = None):
    """X [B,L,d], token_valid [B,L] uint8, pattern_id [B] int32 | None.  Returns (Xp [Tc,d], plan); plan.n_rows[1] > Tc
    says that Tc was too small (the plan is then empty)."""
    assert X.is_contiguous() and token_valid.is_contiguous() and token_valid.dtype == torch.uint8
    B, L, d = X.shape
    if plan is None:
        plan = TokenPackPlan(B, L, token_pack_rows_max(desc) if Tc is None else int(Tc), X.device)
    Xp = torch.empty((plan.Tc, d), dtype=X.dtype, device=X.device) if out is None else out
    rc = lib().sf_token_pack(C.byref(desc), _ptr(X), _ptr(token_valid), _ptr(pattern_id), C.byref(plan.c), _ptr(Xp),
                             _stream())
    _check(rc, "sf_token_pack")
    return Xp, plan


def token_unpack(desc: SfDesc, Yp: torch.Tensor, plan: TokenPackPlan, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Yp [Tc,d] -> Y [B,L,d], zero rows for dropped tokens."""
    assert Yp.is_contiguous()
    Y = torch.empty((plan.B, plan.L, Yp.shape[1]), dtype=Yp.dtype, device=Yp.device) if out is None else out
    _check(lib().sf_token_unpack(C.byref(desc), _ptr(Yp), C.byref(plan.c), _ptr(Y), _stream()), "sf_token_unpack")
    return Y


def encoder_forward_packed(desc: SfDesc, layers: List[CompactLayer], Xp: torch.Tensor, plan: TokenPackPlan,
                           pattern_id: Optional[torch.Tensor], final_ln: Optional[Dict[str, torch.Tensor]] = None,
                           want_sel: bool = False, want_score: bool = False, ws: Optional[torch.Tensor] = None,
                           sample_idx: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None):
    """sf_encoder_forward over packed rows.  Returns (Yp [Tc,d], sel [nl,B,Hq'max,U] | None, score | None)."""
    assert Xp.is_contiguous() and Xp.shape[0] == plan.Tc
    _check_sample(desc, sample_idx, plan.B)
    nl = desc.n_layers
    U = num_active(desc)
    khmax = max(l.k_head for l in layers)
    dev = Xp.device
    Yp = torch.empty_like(Xp) if out is None else out
    sel = torch.full((nl, plan.B, khmax, max(U, 1)), -1, dtype=torch.int32, device=dev) if want_sel else None
    score = torch.full((nl, plan.B, khmax, plan.L), float("-inf"), dtype=torch.float32, device=dev) if want_score else None
    arr = layer_array(layers)
    if ws is None:
        ws = workspace(encoder_packed_workspace_bytes(desc, layers, plan.Tc), dev)
    fg = None if final_ln is None else final_ln["g"]
    fb = None if final_ln is None else final_ln["b"]
    rc = lib().sf_encoder_forward_packed(C.byref(desc), arr, _ptr(Xp), C.byref(plan.c), _ptr(pattern_id), _ptr(sample_idx),
                                         _ptr(fg), _ptr(fb), _ptr(Yp), _ptr(sel), _ptr(score), _ptr(ws), ws.numel(),
                                         _stream())
    _check(rc, "sf_encoder_forward_packed")
    return Yp, sel, score


def encoder_forward_ragged(desc: SfDesc, layers: List[CompactLayer], X: torch.Tensor, pattern_id, key_valid: torch.Tensor,
                           u_active: torch.Tensor, final_ln: Optional[Dict[str, torch.Tensor]] = None,
                           want_sel: bool = False, want_score: bool = False, ws: Optional[torch.Tensor] = None,
                           sample_idx: Optional[torch.Tensor] = None):
    """sf_encoder_forward on a compacted batch: sample b selects min(u_active[b], U) queries per head.
    Returns (Y [B,L,d], sel [nl,B,Hq'max,U] | None, score [nl,B,Hq'max,L] | None)."""
    assert X.is_contiguous()
    _check_sample(desc, sample_idx, X.shape[0])
    B, L, _ = X.shape
    nl = desc.n_layers
    U = num_active(desc)
    khmax = max(l.k_head for l in layers)
    dev = X.device
    Y = torch.empty_like(X)
    sel = torch.full((nl, B, khmax, max(U, 1)), -1, dtype=torch.int32, device=dev) if want_sel else None
    score = torch.full((nl, B, khmax, L), float("-inf"), dtype=torch.float32, device=dev) if want_score else None
    arr = layer_array(layers)
    if ws is None:
        ws = workspace(lib().sf_encoder_workspace_bytes(C.byref(desc), arr), dev)
    fg = None if final_ln is None else final_ln["g"]
    fb = None if final_ln is None else final_ln["b"]
    rc = lib().sf_encoder_forward_ragged(C.byref(desc), arr, _ptr(X), _ptr(pattern_id), _ptr(key_valid), _ptr(u_active),
                                         _ptr(sample_idx), _ptr(fg), _ptr(fb), _ptr(Y), _ptr(sel), _ptr(score), _ptr(ws),
                                         ws.numel(), _stream())
    _check(rc, "sf_encoder_forward_ragged")
    return Y, sel, score


def encoder_forward_fp8ffn(desc: SfDesc, layers: List[CompactLayer], ffn8: List[CompactFfnFp8], X: torch.Tensor,
                           pattern_id: Optional[torch.Tensor] = None, key_valid: Optional[torch.Tensor] = None,
                           final_ln: Optional[Dict[str, torch.Tensor]] = None,
                           forced_sel: Optional[torch.Tensor] = None, want_sel: bool = False, want_codes: bool = False,
                           out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """sf_encoder_forward with every layer's FFN in FP8 arithmetic.  Returns (Y, sel | None) and, with want_codes,
    xq [nl, B*L, d] and a list of hq_l [B*L, Fp8_l]."""
    assert X.is_contiguous() and len(ffn8) == desc.n_layers
    B, L, d = X.shape
    nl = desc.n_layers
    U = num_active(desc)
    khmax = max(l.k_head for l in layers)
    dev = X.device
    Y = torch.empty_like(X) if out is None else out
    sel = torch.full((nl, B, khmax, max(U, 1)), -1, dtype=torch.int32, device=dev) if want_sel else None
    arr = layer_array(layers)
    farr = (SfFfnFp8 * nl)(*[f.struct for f in ffn8])
    if ws is None:
        ws = workspace(lib().sf_encoder_workspace_bytes(C.byref(desc), arr), dev)
    F8max = max(f.Fp8 for f in ffn8)
    xq = torch.empty((nl, B * L, d), dtype=torch.uint8, device=dev) if want_codes else None
    hq = torch.zeros((nl, B * L * F8max), dtype=torch.uint8, device=dev) if want_codes else None
    fg = None if final_ln is None else final_ln["g"]
    fb = None if final_ln is None else final_ln["b"]
    rc = lib().sf_encoder_forward_fp8ffn(C.byref(desc), arr, farr, _ptr(X), _ptr(pattern_id), _ptr(key_valid), None,
                                         _ptr(fg), _ptr(fb), _ptr(forced_sel), _ptr(Y), _ptr(sel if U > 0 else None),
                                         None, _ptr(xq), _ptr(hq), _ptr(ws), ws.numel(), _stream())
    _check(rc, "sf_encoder_forward_fp8ffn")
    if want_codes:
        hql = [hq[l, :B * L * f.Fp8].view(B * L, f.Fp8) for l, f in enumerate(ffn8)]
        return Y, sel, xq, hql
    return Y, sel


# ---------------------------------------------------------- attention projections in FP8 arithmetic
class CompactProjFp8:
    """Q/K/V and output projection weights of one layer as E4M3 codes, compacted for all patterns."""

    def __init__(self, desc: SfDesc, dev, k_head: int, s_qkv: float, so: float, sx1: float, sa: float):
        P, d, dh, Hk = desc.P, desc.d_model, desc.dh, desc.Hk
        self.k_head = int(k_head)
        self.Kp = int(lib().sf_proj_fp8_padded(self.k_head, dh))
        self.Wqkv8 = torch.empty((P, (self.k_head + 2 * Hk) * dh, d), dtype=torch.uint8, device=dev)
        self.WoT8 = torch.empty((P, d, self.Kp), dtype=torch.uint8, device=dev)
        self.struct = SfProjFp8(self.k_head, 0, _ptr(self.Wqkv8), _ptr(self.WoT8), float(s_qkv), float(so),
                                float(sx1), float(sa))


def compact_proj_fp8(desc: SfDesc, layer: int, dense8: Dict[str, torch.Tensor], s_qkv: float, so: float,
                     masks: Dict[str, torch.Tensor], k_head: int, sx1: float, sa: float) -> CompactProjFp8:
    """dense8: Wq [Hq*dh, d], Wk, Wv [Hk*dh, d], Wo [Hq*dh, d] uint8 (E4M3 codes; Wq, Wk, Wv with the one scale
    s_qkv, Wo with so)."""
    for n in ("Wq", "Wk", "Wv", "Wo"):
        assert dense8[n].dtype == torch.uint8 and dense8[n].is_contiguous(), n
    cp = CompactProjFp8(desc, dense8["Wq"].device, k_head, s_qkv, so, sx1, sa)
    nul = C.c_void_p(None)
    ds = SfDenseLayerFp8(_ptr(dense8["Wq"]), _ptr(dense8["Wk"]), _ptr(dense8["Wv"]), _ptr(dense8["Wo"]), nul, nul,
                         float(s_qkv), float(s_qkv), float(s_qkv), float(so), 0.0, 0.0, *([nul] * 10))
    rc = lib().sf_compact_proj_fp8(C.byref(desc), layer, C.byref(ds), _ptr(masks["head_idx"]),
                                   _ptr(masks["group_idx"]), _ptr(masks["n_groups"]), C.byref(cp.struct), _stream())
    _check(rc, "sf_compact_proj_fp8")
    return cp


def encoder_fp8_workspace_bytes(desc: SfDesc, layers: List[CompactLayer]) -> int:
    return int(lib().sf_encoder_fp8_workspace_bytes(C.byref(desc), layer_array(layers)))


def encoder_forward_fp8(desc: SfDesc, layers: List[CompactLayer], X: torch.Tensor,
                        ffn8: Optional[List[CompactFfnFp8]] = None, proj8: Optional[List[CompactProjFp8]] = None,
                        pattern_id: Optional[torch.Tensor] = None, key_valid: Optional[torch.Tensor] = None,
                        final_ln: Optional[Dict[str, torch.Tensor]] = None,
                        forced_sel: Optional[torch.Tensor] = None, want_sel: bool = False, want_codes: bool = False,
                        out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """sf_encoder_forward with the FFNs (ffn8) and / or the attention projections (proj8) in FP8 arithmetic.
    Returns (Y, sel | None) and, with want_codes, a dict of the codes: xq [nl, B*L, d], hq (list of [B*L, Fp8_l]),
    aq [nl, B*L, d], oq (list of [B*L, Kp_l], kept heads in rank order then zero padding); entries of a part that
    is not in FP8 are None."""
    assert X.is_contiguous()
    B, L, d = X.shape
    nl = desc.n_layers
    U = num_active(desc)
    khmax = max(l.k_head for l in layers)
    dev = X.device
    Y = torch.empty_like(X) if out is None else out
    sel = torch.full((nl, B, khmax, max(U, 1)), -1, dtype=torch.int32, device=dev) if want_sel else None
    arr = layer_array(layers)
    farr = None if ffn8 is None else (SfFfnFp8 * nl)(*[f.struct for f in ffn8])
    parr = None if proj8 is None else (SfProjFp8 * nl)(*[p.struct for p in proj8])
    if ws is None:
        ws = workspace(lib().sf_encoder_fp8_workspace_bytes(C.byref(desc), arr), dev)
    xq = hq = aq = oq = None
    if want_codes and ffn8 is not None:
        F8max = max(f.Fp8 for f in ffn8)
        xq = torch.empty((nl, B * L, d), dtype=torch.uint8, device=dev)
        hq = torch.zeros((nl, B * L * F8max), dtype=torch.uint8, device=dev)
    if want_codes and proj8 is not None:
        aq = torch.empty((nl, B * L, d), dtype=torch.uint8, device=dev)
        Kpmax = max(p.Kp for p in proj8)
        oq = torch.zeros((nl, B * L * Kpmax), dtype=torch.uint8, device=dev)
    fg = None if final_ln is None else final_ln["g"]
    fb = None if final_ln is None else final_ln["b"]
    rc = lib().sf_encoder_forward_fp8(C.byref(desc), arr, farr, parr, _ptr(X), _ptr(pattern_id), _ptr(key_valid),
                                      None, _ptr(fg), _ptr(fb), _ptr(forced_sel), _ptr(Y),
                                      _ptr(sel if U > 0 else None), None, _ptr(xq), _ptr(hq), _ptr(aq), _ptr(oq),
                                      _ptr(ws), ws.numel(), _stream())
    _check(rc, "sf_encoder_forward_fp8")
    if not want_codes:
        return Y, sel
    codes = dict(xq=xq, hq=None, aq=aq, oq=None)
    if hq is not None:
        codes["hq"] = [hq[l, :B * L * f.Fp8].view(B * L, f.Fp8) for l, f in enumerate(ffn8)]
    if oq is not None:
        codes["oq"] = [oq[l, :B * L * p.Kp].view(B * L, p.Kp) for l, p in enumerate(proj8)]
    return Y, sel, codes
