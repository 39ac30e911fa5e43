"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
public header declares, computes U like the paper's worked example, and turns
bad arguments into error codes before touching the GPU."""
from __future__ import annotations

import ctypes as C
import os
import re

import pytest

from paper_2604_08971_amd import binding as sf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sentryfuse.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = sorted(set(re.findall(r"\b(sf_[a-z_0-9]+)\s*\(", hdr)))
    assert "sf_encoder_forward" in declared and "sf_sparse_gqa_forward" in declared
    L = sf.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(sf.EXPORTS) == declared
    # the FP16 build of the same sources exports the same entry points
    with sf.use_half("f16"):
        L16 = sf.lib()
        assert L16 is not L
        for name in declared:
            assert hasattr(L16, name), name
        # each build takes 16-bit models of its own type only (checked on the host, before any launch)
        d16, dbf = sf.make_desc(1, 64, 64, 4, 2, 16, 128, dtype=sf.SF_F16), sf.make_desc(1, 64, 64, 4, 2, 16, 128, dtype=sf.SF_BF16)
        assert L16.sf_num_active(C.byref(d16)) > 0 and L16.sf_num_active(C.byref(dbf)) == -3
        assert L.sf_num_active(C.byref(dbf)) > 0 and L.sf_num_active(C.byref(d16)) == -3
        assert L16.sf_num_active(C.byref(sf.make_desc(1, 64, 64, 4, 2, 16, 128, dtype=sf.SF_F32))) > 0


def test_struct_layout_matches_header():
    assert C.sizeof(sf.SfDesc) == 18 * 4
    assert C.sizeof(sf.SfStrides) == 24
    assert C.sizeof(sf.SfDenseLayer) == 16 * 8
    assert C.sizeof(sf.SfCompactLayer) == 8 + 14 * 8
    assert C.sizeof(sf.SfMoeDense) == 8 * 8
    assert C.sizeof(sf.SfMoeCompact) == 16 + 9 * 8
    assert C.sizeof(sf.SfGateParams) == 16 + 6 * 8
    assert C.sizeof(sf.SfDenseLayerFp8) == 6 * 8 + 6 * 4 + 10 * 8
    assert C.sizeof(sf.SfFfnFp8) == 8 + 6 * 8 + 4 * 4
    assert C.sizeof(sf.SfProjFp8) == 8 + 2 * 8 + 4 * 4


def test_num_active_matches_paper_example():
    # Sec. 4.4: T = 128, c = 5 gives U of about 25 (natural log)
    assert sf.num_active(sf.make_desc(1, 128, 64, 8, 2, 8, 64)) == 25
    for L, U in ((48, 20), (384, 30), (480, 35), (512, 35), (4096, 45), (1, 0), (3, 3)):
        assert sf.num_active(sf.make_desc(1, L, 64, 8, 2, 8, 64)) == U
    assert sf.num_active(sf.make_desc(1, 128, 64, 8, 2, 8, 64, U_override=500)) == 128
    assert sf.num_active(sf.make_desc(1, 128, 64, 8, 2, 8, 64, U_override=0)) == 0
    assert sf.num_active(sf.make_desc(1, 128, 64, 8, 2, 8, 64, c_factor=2)) == 10
    assert sf.ffn_padded(sf.make_desc(1, 128, 64, 8, 2, 8, 3072), 2150) == 2176
    assert sf.ffn_padded(sf.make_desc(1, 128, 64, 8, 2, 8, 3072, ffn_pad=128), 2150) == 2176


@pytest.mark.parametrize("kw,code", [
    (dict(Hq=8, Hk=3), -1), (dict(B=0), -1), (dict(L=0), -1), (dict(dtype=7), -3), (dict(act=9), -3),
    (dict(ffn_pad=48), -2), (dict(d_model=60, dtype=sf.SF_BF16), -2), (dict(dh=12, dtype=sf.SF_BF16), -2),
])
def test_bad_descriptor_is_rejected(kw, code):
    base = dict(B=1, L=16, d_model=64, Hq=8, Hk=2, dh=8, d_ff=64, dtype=sf.SF_F32)
    base.update(kw)
    d = sf.make_desc(**base)
    assert sf.lib().sf_num_active(C.byref(d)) == code
    assert len(sf.lib().sf_last_error()) > 0
    d2 = sf.make_desc(1, 16, 64, 8, 2, 8, 64)
    d2.struct_size = 12
    assert sf.lib().sf_num_active(C.byref(d2)) == -1


def test_null_and_range_errors_before_any_launch():
    L = sf.lib()
    d = sf.make_desc(2, 16, 64, 8, 2, 8, 64, dtype=sf.SF_F32)
    assert L.sf_gate_scores_to_masks(C.byref(d), *([None] * 12)) == -1
    assert L.sf_encoder_forward(C.byref(d), None, None, None, None, None, None, None, None, None, None, None,
                                None, 0, None) == -1
    z = sf.SfStrides(0, 0, 0)
    assert L.sf_sparse_gqa_forward(C.byref(d), 4, 2, None, z, None, z, None, z, 0, None, None, None, None, None,
                                   None, 32, None, None, None, 0, None) == -1
    assert L.sf_sparse_gqa_forward(C.byref(d), 0, 2, None, z, None, z, None, z, 0, None, None, None, None, None,
                                   None, 32, None, None, None, 0, None) == -1
    d_bad = sf.make_desc(2, 16, 64, 8, 2, 8, 64, dtype=sf.SF_F32, n_sample=5000)
    assert L.sf_num_active(C.byref(d_bad)) == -1
    d_s = sf.make_desc(2, 16, 64, 8, 2, 8, 64, dtype=sf.SF_F32, n_sample=7)
    assert L.sf_sparse_gqa_workspace_bytes(C.byref(d_s), 4, 2) > L.sf_sparse_gqa_workspace_bytes(C.byref(d), 4, 2)
    assert L.sf_pruned_ffn_forward(C.byref(d), None, None, None, 1, 1, None, None, 0, None) == -1
    assert L.sf_sparse_gqa_workspace_bytes(C.byref(d), 4, 2) > 0
    assert L.sf_pruned_ffn_workspace_bytes(C.byref(d), 0) == 0
    cl = sf.SfCompactLayer()
    cl.k_head, cl.k_ffn = 9, 10          # more heads than the model has
    assert L.sf_encoder_workspace_bytes(C.byref(d), C.byref(cl)) == 0
    cl.k_head = 4
    assert L.sf_encoder_workspace_bytes(C.byref(d), C.byref(cl)) > 0
    # Sparse-MoE block: structure checks come before any launch
    m = sf.SfMoeCompact()
    m.n_experts, m.top_k, m.k_ffn_max = 4, 5, 32          # top_k > E
    assert L.sf_moe_ffn_workspace_bytes(C.byref(d), C.byref(m)) == 0
    m.top_k = 2
    assert L.sf_moe_ffn_workspace_bytes(C.byref(d), C.byref(m)) == 0      # no device keep counts
    m.k_ffn = 256
    assert L.sf_moe_ffn_workspace_bytes(C.byref(d), C.byref(m)) > 0
    m.k_ffn_max = 65                                      # more channels than the model has
    assert L.sf_moe_ffn_workspace_bytes(C.byref(d), C.byref(m)) == 0
    m.k_ffn_max = 32
    assert L.sf_moe_ffn_forward(C.byref(d), C.byref(m), None, None, 1, 1, None, None, None, None, None, None, 0,
                                None) == -1
    assert L.sf_compact_moe_experts(C.byref(d), None, None, None, C.byref(m), None) == -1
    # SentryGate entry points
    gp = sf.SfGateParams()
    gp.n_modalities, gp.hidden, gp.nonlin = 3, 16, 0
    assert L.sf_gate_eval(C.byref(d), C.byref(gp), None, None, None, None) == -1
    one = C.c_void_p(256)
    gp.Wa = gp.Wb = gp.zeta = gp.gamma = 256
    gp.hidden = 5000
    assert L.sf_gate_eval(C.byref(d), C.byref(gp), one, one, one, None) == -1
    gp.hidden, gp.nonlin = 16, 7
    assert L.sf_gate_eval(C.byref(d), C.byref(gp), one, one, one, None) == -3
    c1 = (C.c_int64 * 1)(5)
    neg = (C.c_int64 * 1)(-5)
    cp = lambda a: C.cast(a, C.c_void_p)
    assert L.sf_budget_search(C.byref(d), one, one, 0, cp(c1), cp(c1), cp(c1), 0, 10, None, one, one, one, one, None) == -1
    assert L.sf_budget_search(C.byref(d), one, one, 3, cp(c1), cp(c1), cp(c1), 0, 10, one, one, one, one, one, None) == -1
    assert L.sf_budget_search(C.byref(d), one, one, 0, cp(c1), cp(neg), cp(c1), 0, 10, one, one, one, one, one, None) == -1
    d8 = sf.SfDenseLayerFp8()
    cl8 = sf.SfCompactLayer()
    cl8.k_head, cl8.k_ffn = 4, 10
    assert L.sf_compact_heads_channels_fp8(C.byref(d), 0, C.byref(d8), one, one, one, one, C.byref(cl8), None) == -1   # NULL matrices
    assert L.sf_compact_heads_channels_fp8(C.byref(d), 5, C.byref(d8), one, one, one, one, C.byref(cl8), None) == -1   # layer out of range
    # FP8 arithmetic of the FFN: every check comes before the first launch
    assert L.sf_ffn_fp8_padded(2150) == 2176 and L.sf_ffn_fp8_padded(128) == 128 and L.sf_ffn_fp8_padded(129) == 256
    assert L.sf_ffn_fp8_padded(0) == 0
    assert L.sf_quantize_fp8(None, sf.SF_F32, 8, 1.0, None, None) == -1
    assert L.sf_quantize_fp8(one, 7, 8, 1.0, one, None) == -1
    assert L.sf_quantize_fp8(one, sf.SF_F32, 8, 0.0, one, None) == -1
    assert L.sf_quantize_fp8(one, sf.SF_F32, 8, float("inf"), one, None) == -1
    assert L.sf_quantize_fp8(C.c_void_p(260), sf.SF_F32, 8, 1.0, one, None) == -1          # misaligned
    assert L.sf_quantize_fp8(None, sf.SF_F32, 0, 1.0, None, None) == 0                      # nothing to do
    f8 = sf.SfFfnFp8()
    f8.k_ffn, f8.s1, f8.s2, f8.sx, f8.sh = 200, 1.0, 1.0, 1.0, 1.0
    f8.W1q = f8.W2Tq = 256
    d8ok = sf.make_desc(1, 256, 256, 8, 2, 8, 512, dtype=sf.SF_BF16)
    args = (one, None, 1, 1, C.c_void_p(512), None, None, None, 0, None)
    assert L.sf_pruned_ffn_fp8_forward(C.byref(d8ok), C.byref(f8), *args) == -4            # no workspace
    assert L.sf_pruned_ffn_fp8_forward(C.byref(d), C.byref(f8), *args) in (-2, -3)          # fp32 descriptor
    for kw in (dict(L=100), dict(d_model=192), dict(d_model=200)):
        base = dict(B=1, L=256, d_model=256, Hq=8, Hk=2, dh=8, d_ff=512, dtype=sf.SF_BF16)
        base.update(kw)
        assert L.sf_pruned_ffn_fp8_forward(C.byref(sf.make_desc(**base)), C.byref(f8), *args) in (-2, -3)
    f8.k_ffn = 100
    assert L.sf_pruned_ffn_fp8_forward(C.byref(d8ok), C.byref(f8), *args) == -3            # too few channels
    f8.k_ffn, f8.sh = 200, -1.0
    assert L.sf_pruned_ffn_fp8_forward(C.byref(d8ok), C.byref(f8), *args) == -1
    assert L.sf_compact_ffn_fp8(C.byref(d8ok), 0, C.byref(d8), one, C.byref(f8), None) == -1   # NULL dense matrices
    assert L.sf_compact_ffn_fp8(C.byref(d8ok), 3, C.byref(d8), one, C.byref(f8), None) == -1   # layer out of range
    assert L.sf_pruned_ffn_fp8_workspace_bytes(C.byref(d8ok), 200) == 256 * 256 + 256 * 256
    # encoder with FP8 FFNs: the checks of every layer's FFN come before anything is enqueued
    f8.k_ffn, f8.sh = 200, 1.0
    cl8f = sf.SfCompactLayer()
    cl8f.k_head, cl8f.k_ffn = 4, 200
    eargs = (one, None, None, None, None, None, None, C.c_void_p(512), None, None, None, None, None, 0, None)
    assert L.sf_encoder_forward_fp8ffn(C.byref(d8ok), C.byref(cl8f), None, *eargs) == -1          # no FFN array
    assert L.sf_encoder_forward_fp8ffn(C.byref(d), C.byref(cl8f), C.byref(f8), *eargs) in (-2, -3)  # fp32 descriptor
    cl8f.k_ffn = 300
    assert L.sf_encoder_forward_fp8ffn(C.byref(d8ok), C.byref(cl8f), C.byref(f8), *eargs) == -1   # k_ffn mismatch
    # encoder with FP8 projections: checked before anything is enqueued
    cl8f.k_ffn = 200
    pj = sf.SfProjFp8()
    pj.k_head, pj.s_qkv, pj.so, pj.sx1, pj.sa = 4, 1.0, 1.0, 1.0, 1.0
    pj.Wqkv8 = pj.WoT8 = 256
    dp = sf.make_desc(1, 256, 256, 8, 2, 32, 512, dtype=sf.SF_BF16)
    pargs = eargs[:12] + (None, None) + eargs[12:]
    assert L.sf_encoder_forward_fp8(C.byref(dp), C.byref(cl8f), None, None, *pargs) == -1         # neither part in FP8
    assert L.sf_encoder_forward_fp8(C.byref(d), C.byref(cl8f), None, C.byref(pj), *pargs) in (-2, -3)   # fp32 descriptor
    pj.k_head = 3
    assert L.sf_encoder_forward_fp8(C.byref(dp), C.byref(cl8f), None, C.byref(pj), *pargs) == -1  # k_head mismatch
    assert L.sf_proj_fp8_padded(3, 32) == 128 and L.sf_proj_fp8_padded(8, 64) == 512 and L.sf_proj_fp8_padded(5, 64) == 384
    assert L.sf_proj_fp8_padded(0, 64) == 0
    dnarrow = sf.make_desc(1, 256, 256, 2, 1, 32, 512, dtype=sf.SF_BF16)
    pj.k_head, cl8f.k_head = 1, 1
    assert L.sf_encoder_forward_fp8(C.byref(dnarrow), C.byref(cl8f), None, C.byref(pj), *pargs) == -3  # 96 Q/K/V features
    pj.k_head, cl8f.k_head, pj.sa = 4, 4, 0.0
    assert L.sf_encoder_forward_fp8(C.byref(dp), C.byref(cl8f), None, C.byref(pj), *pargs) == -1
    pj.sa = 1.0
    d8.sq, d8.sk, d8.sv, d8.so = 1.0, 1.0, 1.0, 1.0
    assert L.sf_compact_proj_fp8(C.byref(dp), 0, C.byref(d8), one, one, one, C.byref(pj), None) == -1   # NULL dense matrices
    assert L.sf_compact_proj_fp8(C.byref(dp), 5, C.byref(d8), one, one, one, C.byref(pj), None) == -1   # layer out of range
    assert L.sf_encoder_fp8_workspace_bytes(C.byref(dp), C.byref(cl8f)) > L.sf_encoder_workspace_bytes(C.byref(dp), C.byref(cl8f))
    # FP16-stored weights
    assert L.sf_compact_heads_channels_f16(C.byref(d), 0, None, one, one, one, one, C.byref(cl8), None) == -1
    dl16 = sf.SfDenseLayer()
    assert L.sf_compact_heads_channels_f16(C.byref(d), 0, C.byref(dl16), one, one, one, one, C.byref(cl8), None) == -1
    # token compaction
    assert L.sf_token_compact(C.byref(d), None, one, 8, one, one, one, one, one, one, None) == -1
    assert L.sf_token_compact(C.byref(d), one, one, 0, C.c_void_p(512), one, one, one, one, one, None) == -1      # Lc < 1
    assert L.sf_token_compact(C.byref(d), one, one, d.L + 1, C.c_void_p(512), one, one, one, one, one, None) == -1
    assert L.sf_token_compact(C.byref(d), one, one, 8, one, one, one, one, one, one, None) == -1                  # Xc aliases X
    assert L.sf_token_scatter(C.byref(d), one, None, 8, C.c_void_p(512), None) == -1
    assert L.sf_token_scatter(C.byref(d), one, one, 8, one, None) == -1                                           # Y aliases Yc
    cl9 = sf.SfCompactLayer()
    assert L.sf_encoder_forward_ragged(C.byref(d), C.byref(cl9), one, None, one, None, None, None, None,
                                       C.c_void_p(512), None, None, None, 0, None) == -1                          # no u_active
    du = sf.make_desc(1, 16, 64, 8, 2, 8, 64, dtype=sf.SF_F32, U_override=16)
    assert L.sf_encoder_forward_ragged(C.byref(du), C.byref(cl9), one, None, one, one, None, None, None,
                                       C.c_void_p(512), None, None, None, 0, None) == -3                          # U >= L
    # host-side keep counts out of range
    kh, kf = (C.c_int32 * 1)(9), (C.c_int32 * 1)(3)
    one = C.c_void_p(256)                 # never dereferenced: the count check comes first
    assert L.sf_gate_scores_to_masks(C.byref(d), one, one, C.cast(kh, C.c_void_p), C.cast(kf, C.c_void_p),
                                     one, one, one, one, one, one, one, None) == -1


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the public header compiles as C99 with no C++ or HIP types."""
    import subprocess
    src = tmp_path / "hdr.c"
    src.write_text('#include "sentryfuse.h"\nint main(void) { sf_desc d; (void)d; return (int)sizeof(sf_moe_compact) == 0; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                           "-fsyntax-only", str(src)])
