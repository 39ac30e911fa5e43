"""GPU parity: the HIP library (through the C ABI) against the CPU oracle,
element by element on the same seeded inputs.

Bar: masks, kept-index lists and compacted weights bit-exact; outputs within
max |a-b| / max(1,|b|) <= 1e-5 (fp32) or 2e-2 (bf16 inputs, fp32 accumulate).
The active-query choice is a floating-point decision: the GPU's choice must be
within a margin of the oracle's threshold score, and outputs are compared with
the oracle re-run on the GPU's choice.
"""
from __future__ import annotations

import math

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as orc
from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W
from gpu_utils import ORACLE_MODE, SF_DTYPE, DeviceModel, selection_report, to_dev, to_host
from helpers import compact_packs, compact_weights, err_metric, make_wl, oracle_masks

pytestmark = pytest.mark.gpu

# bf16: 5 units of 2^-8 (the spacing relative to the larger of 1 and the value); binary16 has three more bits:
# 8 units of 2^-11
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 4e-3}
EPS_SEL_OP = {"f32": 1e-5, "bf16": 1e-4, "f16": 1e-4}       # sparse_gqa_forward on identical inputs
EPS_SEL_ENC = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}      # inside the encoder (inputs differ by 16-bit rounding)


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ a1: masks
MASK_KEYS = ("head_mask", "ffn_mask", "head_idx", "ffn_idx", "group_idx", "n_groups", "head_group")


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_masks_bit_exact_on_configs(name):
    _say(f"masks {name}")
    wl = make_wl(W.CONFIGS[name], with_x=False)
    ref = oracle_masks(wl)
    desc = sf.make_desc(1, wl.spec.L, wl.spec.d, wl.spec.Hq, wl.spec.Hk, wl.spec.dh, wl.spec.F,
                        wl.spec.n_layers, wl.P, sf.SF_F32)
    got = sf.gate_scores_to_masks(desc, to_dev(wl.g_head, "f32"), to_dev(wl.g_ffn, "f32"), wl.k_head, wl.k_ffn)
    torch.cuda.synchronize()
    for k in MASK_KEYS:
        assert np.array_equal(to_host(got[k]), ref[k]), k


@pytest.mark.parametrize("Hq,Hk,F,kh,kf", [(8, 2, 257, 3, 100), (64, 8, 16384, 17, 9000), (1, 1, 1, 1, 1),
                                           (12, 4, 3000, 12, 3000), (6, 3, 33, 1, 1)])
def test_masks_ties_and_edges(Hq, Hk, F, kh, kf):
    _say(f"masks ties Hq={Hq} F={F}")
    rng = np.random.default_rng(Hq * 1000 + F)
    nl, P = 2, 3
    g_head = (rng.integers(0, 3, (nl, P, Hq)) / 2).astype(np.float32)            # heavy ties
    g_ffn = (rng.integers(0, 7, (nl, P, F)) / 8 - 0.25).astype(np.float32)       # ties, negatives, +-0
    g_ffn[0, 0, : F // 2] = -0.0
    ref = orc.gate_scores_to_masks(g_head, g_ffn, [kh, Hq], [kf, F], Hk)
    desc = sf.make_desc(1, 8, 8, Hq, Hk, 8, F, nl, P, sf.SF_F32)
    got = sf.gate_scores_to_masks(desc, to_dev(g_head, "f32"), to_dev(g_ffn, "f32"), [kh, Hq], [kf, F])
    torch.cuda.synchronize()
    for k in MASK_KEYS:
        assert np.array_equal(to_host(got[k]), ref[k]), k


# ------------------------------------------------------------- a2: compaction
def _check_compaction(wl, dm, ref_masks):
    s = wl.spec
    for l in range(s.n_layers):
        cl = dm.layers[l]
        kh, kf, Fp = int(wl.k_head[l]), int(wl.k_ffn[l]), cl.Fp
        assert Fp % 64 == 0 and Fp >= kf and Fp - kf < 64
        for p in range(wl.P):
            c, _, ng, _ = compact_weights(wl, ref_masks, l, p)
            dh, Hk, d = s.dh, s.Hk, s.d
            Wqkv = to_host(cl.Wqkv[p]); bqkv = to_host(cl.bqkv[p])
            nq = kh * dh
            assert np.array_equal(Wqkv[:nq], c["Wq"]) and np.array_equal(bqkv[:nq], c["bq"])
            assert np.array_equal(Wqkv[nq:nq + ng * dh], c["Wk"]) and np.array_equal(bqkv[nq:nq + ng * dh], c["bk"])
            assert not Wqkv[nq + ng * dh: nq + Hk * dh].any() and not bqkv[nq + ng * dh: nq + Hk * dh].any()
            v0 = nq + Hk * dh
            assert np.array_equal(Wqkv[v0:v0 + ng * dh], c["Wv"]) and np.array_equal(bqkv[v0:v0 + ng * dh], c["bv"])
            assert not Wqkv[v0 + ng * dh:].any() and not bqkv[v0 + ng * dh:].any()
            assert np.array_equal(to_host(cl.WoT[p]), c["Wo"].T)
            W1 = to_host(cl.W1[p]); b1 = to_host(cl.b1[p]); W2T = to_host(cl.W2T[p])
            assert np.array_equal(W1[:kf], c["W1"]) and not W1[kf:].any()
            assert np.array_equal(b1[:kf], c["b1"]) and not b1[kf:].any()
            assert np.array_equal(W2T[:, :kf], c["W2"].T) and not W2T[:, kf:].any()


def test_key_valid_matches_oracle():
    # presence masks -> allowed keys (Sec. 4.2 / 4.4): the library's derivation on the device against the oracle's
    # own, bit for bit: the five workloads, ragged small ones with fusion tokens, rows with a single modality left,
    # interleaved modalities, M = 0 (modality-free tokens only)
    _say("key_valid from presence")
    cases = [(W.make_workload(W.CONFIGS[n], with_x=False).presence, W.make_workload(W.CONFIGS[n], with_x=False).tok_modality)
             for n in ("C1", "C2", "C3", "C4", "C5")]
    for seed in range(3):
        wl = W.make_workload(W.small_spec(B=9, seg=(7, 5, 9, 2), extra=3, seed=seed, dropout="bernoulli:0.5"), with_x=False)
        cases.append((wl.presence, wl.tok_modality))
    rng = np.random.default_rng(3)
    tm = rng.integers(-1, 5, size=1031).astype(np.int32)                  # interleaved, ragged length
    pres = (rng.random((37, 5)) < 0.4).astype(np.uint8)
    pres[3] = 0; pres[3, 2] = 1                                           # all but one absent
    pres[4] = 1                                                           # nothing absent
    pres[5] = 0                                                           # only the modality-free tokens remain
    pres[6] = 0; pres[6, 0] = 200                                         # any non-zero byte = present
    cases.append((pres, tm))
    cases.append((np.zeros((2, 0), np.uint8), np.full(5, -1, np.int32)))  # M = 0
    for pres, tm in cases:
        ref = orc.key_valid(pres, tm)
        got = sf.presence_to_key_valid(torch.from_numpy(pres).cuda(), torch.from_numpy(tm).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(to_host(got), ref), (pres.shape, tm.shape)
    # DeviceModel hands the library's own mask to the encoder; the tests hand the oracle's to the oracle
    wl = make_wl(W.CONFIGS["C3"], with_x=False)
    wl.x = np.zeros((wl.presence.shape[0], wl.spec.L, wl.spec.d), np.float32)
    assert np.array_equal(to_host(DeviceModel(wl).key_valid), wl.key_valid)
    with pytest.raises(sf.SentryFuseError):
        sf.presence_to_key_valid(torch.zeros((1, 65), dtype=torch.uint8).cuda(), torch.zeros(4, dtype=torch.int32).cuda())


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_compaction_bit_exact_on_configs(name):
    _say(f"compaction {name}")
    wl = make_wl(W.CONFIGS[name], with_x=False)
    ref = oracle_masks(wl)
    # the numpy slicing used as reference agrees with the oracle's own row gather
    c, kh, ng, _ = compact_weights(wl, ref, 0, 0)
    assert np.array_equal(orc.gather_rows(wl.layers[0]["W1"], ref["ffn_idx"][0, 0, :wl.k_ffn[0]]), c["W1"])
    assert np.array_equal(orc.gather_rows(wl.layers[0]["Wq"], ref["head_idx"][0, 0, :kh], block=wl.spec.dh), c["Wq"])
    wl.x = np.zeros((1, wl.spec.L, wl.spec.d), np.float32)
    wl.pattern_id = wl.pattern_id[:1]
    wl.presence = wl.presence[:1]
    if wl.key_valid is not None:
        wl.key_valid = wl.key_valid[:1]
    dm = DeviceModel(wl).build_plan()
    torch.cuda.synchronize()
    _check_compaction(wl, dm, ref)


def test_compaction_keep_all_is_identity():
    spec = W.small_spec(dtype="bf16", d=64, dh=32, Hq=4, Hk=2, F=128, head_keep=1.0, ffn_keep=1.0, nl=1)
    wl = make_wl(spec)
    dm = DeviceModel(wl).build_plan()
    torch.cuda.synchronize()
    cl = dm.layers[0]
    for p in range(wl.P):
        w = wl.layers[0]
        assert np.array_equal(to_host(cl.Wqkv[p]), np.concatenate([w["Wq"], w["Wk"], w["Wv"]]))
        assert np.array_equal(to_host(cl.W1[p]), w["W1"]) and np.array_equal(to_host(cl.W2T[p]), w["W2"].T)
        assert np.array_equal(to_host(cl.WoT[p]), w["Wo"].T)


# -------------------------------------------------- FP8 (OCP E4M3) weight storage
W8 = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")


def _quantise_fp8(wl):
    """Per-matrix scale = amax / 448 and PyTorch's float8_e4m3fn cast as the (library) quantiser.  Returns the
    codes, the scales, and a copy of the workload whose dense weights are the ORACLE's dequantised values."""
    import copy
    bf = wl.spec.dtype == "bf16"
    codes, scales = [], []
    wl2 = copy.copy(wl)
    wl2.layers = []
    for lw in wl.layers:
        q, sc, lw2 = {}, {}, dict(lw)
        for n in W8:
            w = lw[n].astype(np.float32)
            sc[n] = float(np.float32(np.abs(w).max() / 448.0))
            q[n] = torch.from_numpy(w / np.float32(sc[n])).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            assert not ((q[n] & 0x7F) == 0x7F).any()
            lw2[n] = orc.dequant_fp8(q[n], sc[n], bf).astype(np.float32)
        codes.append(q); scales.append(sc); wl2.layers.append(lw2)
    return codes, scales, wl2


def _fp8_case(wl):
    s = wl.spec
    codes, scales, wl2 = _quantise_fp8(wl)
    dm = DeviceModel(wl2).build_plan()                       # the 16/32-bit path on the oracle's dequantised weights
    for l in range(s.n_layers):
        d8 = {n: (to_dev(codes[l][n], s.dtype) if n in W8 else dm.dense[l][n]) for n in dm.dense[l]}
        cl = sf.compact_heads_channels_fp8(dm.desc, l, d8, scales[l], dm.masks, int(wl.k_head[l]), int(wl.k_ffn[l]))
        torch.cuda.synchronize()
        ref = dm.layers[l]
        for n in ("Wqkv", "bqkv", "WoT", "W1", "b1", "W2T"):
            a, b = getattr(cl, n), getattr(ref, n)
            assert (a is None) == (b is None), n
            if a is not None:
                assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                                   b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32)), (l, n)
        dm.layers[l] = cl                                    # the forward below runs on the FP8-sourced buffers
    return wl2, dm


@pytest.mark.parametrize("kw", [dict(dtype="f32"), dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=3),
                                dict(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=320, seg=(100, 133, 64), extra=3, B=4, act=1,
                                     dropout="upto:2")])
def test_fp8_weight_storage_small(kw):
    """Compaction from FP8 storage is bit-identical to compaction of the oracle's dequantised weights, and the
    encoder on those buffers matches the oracle run on the dequantised weights."""
    _say(f"fp8 storage {kw}")
    wl = make_wl(W.small_spec(**kw))
    wl2, dm = _fp8_case(wl)
    y8 = dm.forward()[0].clone()
    torch.cuda.synchronize()
    _encoder_parity(wl2)
    dm2 = DeviceModel(wl2).build_plan()
    assert torch.equal(y8, dm2.forward()[0])


@pytest.mark.parametrize("name", ["C2", "C5"])
def test_fp8_weight_storage_full_size(name):
    _say(f"fp8 storage {name}")
    _fp8_case(make_wl(W.CONFIGS[name]))


def _f16_case(wl):
    """Weights stored as binary16 (numpy's float16 cast as the offline quantiser): compaction from that storage is
    bit-identical to compaction of the oracle's dequantised weights."""
    import copy
    s = wl.spec
    bf = s.dtype == "bf16"
    wl2 = copy.copy(wl)
    wl2.layers, bits = [], []
    for lw in wl.layers:
        lw2, q = dict(lw), {}
        for n in W8:
            q[n] = lw[n].astype(np.float16).view(np.uint16)
            lw2[n] = orc.dequant_f16(q[n], bf).astype(np.float32)
        wl2.layers.append(lw2); bits.append(q)
    dm = DeviceModel(wl2).build_plan()
    for l in range(s.n_layers):
        d16 = {n: (torch.from_numpy(bits[l][n].view(np.float16)).cuda() if n in W8 else dm.dense[l][n]) for n in dm.dense[l]}
        cl = sf.compact_heads_channels_f16(dm.desc, l, d16, dm.masks, int(wl.k_head[l]), int(wl.k_ffn[l]))
        torch.cuda.synchronize()
        ref = dm.layers[l]
        for n in ("Wqkv", "bqkv", "WoT", "W1", "b1", "W2T"):
            a, b = getattr(cl, n), getattr(ref, n)
            assert (a is None) == (b is None), n
            if a is not None:
                assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                                   b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32)), (l, n)
        dm.layers[l] = cl
    return wl2, dm


@pytest.mark.parametrize("kw", [dict(dtype="f32"), dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=3)])
def test_f16_weight_storage_small(kw):
    _say(f"f16 storage {kw}")
    wl2, dm = _f16_case(make_wl(W.small_spec(**kw)))
    y16 = dm.forward()[0].clone()
    torch.cuda.synchronize()
    _encoder_parity(wl2)                                     # the oracle on the dequantised weights
    assert torch.equal(y16, DeviceModel(wl2).build_plan().forward()[0])


@pytest.mark.parametrize("name", ["C1", "C5"])
def test_f16_weight_storage_full_size(name):
    _say(f"f16 storage {name}")
    _f16_case(make_wl(W.CONFIGS[name]))


# -------------------------------------------------- SentryGate: Eq. (1) and the global threshold
def _gate_case(nl, M, Hq, Hk, F, Hd, nonlin, seed):
    gp = W.make_gate_params(nl, M, Hq, F, Hd, seed)
    bits = np.arange(1, 2 ** M, dtype=np.int32)                   # every pattern with at least one modality
    P = len(bits)
    desc = sf.make_desc(1, 8, 8, Hq, Hk, 8, F, nl, P, sf.SF_F32)
    gh, gf = sf.gate_eval(desc, {k: to_dev(v, "f32") for k, v in gp.items()}, to_dev(bits, "f32"), nonlin)
    torch.cuda.synchronize()
    rh, rf = orc.gate_eval(gp, bits, Hq, nonlin)
    gh_h, gf_h = to_host(gh), to_host(gf)
    # fp32 dot products of Hd terms and one expf against fp64; d sigmoid / dz <= 1/4.  The rounding of the
    # dot product grows with Hd (terms of size ~|h|/sqrt(Hd), gamma <= 2): 1e-6 up to 64 terms, 1e-5 beyond
    tol = 1e-6 if Hd <= 64 else 1e-5
    assert np.max(np.abs(gh_h - rh)) <= tol and np.max(np.abs(gf_h - rf)) <= tol
    return desc, gh, gf, gh_h, gf_h, P


@pytest.mark.parametrize("nl,M,Hq,Hk,F,Hd,nonlin", [(2, 3, 4, 2, 48, 16, 0), (1, 2, 12, 4, 3072, 64, 1),
                                                     (6, 3, 8, 2, 2048, 13, 0), (3, 4, 8, 4, 300, 7, 1),
                                                     (1, 1, 1, 1, 1, 1, 0), (2, 5, 64, 8, 1000, 1024, 0)])
def test_gate_eval_parity(nl, M, Hq, Hk, F, Hd, nonlin):
    _say(f"gate_eval nl={nl} M={M} Hq={Hq} F={F} Hd={Hd} nonlin={nonlin}")
    _gate_case(nl, M, Hq, Hk, F, Hd, nonlin, seed=nl * 100 + Hd)


def _budget_check(desc, gh, gf, gh_h, gf_h, p, Hk, costs, fixed, budget):
    got = sf.budget_search(desc, gh, gf, p, *costs, fixed, budget)
    torch.cuda.synchronize()
    ref = orc.budget_search(gh_h[:, p], gf_h[:, p], Hk, *costs, fixed, budget)      # the same fp32 scores on both sides
    tau = to_host(got["tau"])[0]
    assert bool(to_host(got["feasible"])[0]) == ref["feasible"], budget
    assert (np.isinf(tau) and np.isinf(ref["tau"])) or tau == ref["tau"], (budget, tau, ref["tau"])
    assert np.array_equal(to_host(got["k_head"]), ref["k_head"]) and np.array_equal(to_host(got["k_ffn"]), ref["k_ffn"])
    assert int(to_host(got["cost"])[0]) == ref["cost"]
    return got, ref


@pytest.mark.parametrize("nl,M,Hq,Hk,F", [(2, 3, 4, 2, 48), (6, 3, 8, 2, 2048), (4, 2, 32, 8, 4096), (1, 2, 12, 4, 3072)])
def test_budget_search_parity(nl, M, Hq, Hk, F):
    _say(f"budget_search nl={nl} Hq={Hq} F={F}")
    desc, gh, gf, gh_h, gf_h, P = _gate_case(nl, M, Hq, Hk, F, 16, 0, seed=nl + F)
    rng = np.random.default_rng(F)
    costs = (rng.integers(1000, 5000, nl).tolist(), rng.integers(500, 2000, nl).tolist(), rng.integers(5, 40, nl).tolist())
    fixed = 12345
    dense = fixed + sum(Hq * costs[0][l] + Hk * costs[1][l] + F * costs[2][l] for l in range(nl))
    floor = fixed + sum(costs[0][l] + costs[1][l] + costs[2][l] for l in range(nl))
    for p in sorted({0, P // 2, P - 1}):
        for budget in (dense, dense - 1, int(0.7 * dense), int(0.5 * dense), int(0.2 * dense), floor + 1, floor, floor - 1, 0):
            got, ref = _budget_check(desc, gh, gf, gh_h, gf_h, p, Hk, costs, fixed, budget)
        # the counts drive the mask builder: its top-k with these counts is the set of units >= tau
        got, ref = _budget_check(desc, gh, gf, gh_h, gf_h, p, Hk, costs, fixed, int(0.6 * dense))
        masks = sf.gate_scores_to_masks(desc, gh, gf, ref["k_head"].tolist(), ref["k_ffn"].tolist())
        torch.cuda.synchronize()
        hm, fm = to_host(masks["head_mask"])[:, p].astype(bool), to_host(masks["ffn_mask"])[:, p].astype(bool)
        for l in range(nl):
            if (gh_h[l, p] >= ref["tau"]).any():
                assert np.array_equal(hm[l], gh_h[l, p] >= ref["tau"])
            if (gf_h[l, p] >= ref["tau"]).any():
                assert np.array_equal(fm[l], gf_h[l, p] >= ref["tau"])


def test_budget_search_ties_and_signs():
    """Scores given directly (not from Eq. (1)): heavy ties, negatives, both zeros, a tie at the maximum."""
    nl, Hq, Hk, F, P = 3, 6, 3, 257, 2
    rng = np.random.default_rng(5)
    gh_h = (rng.integers(-2, 3, (nl, P, Hq)) / 2).astype(np.float32)
    gf_h = (rng.integers(-4, 5, (nl, P, F)) / 8).astype(np.float32)
    gf_h[0, 0, : F // 3] = -0.0
    gf_h[2, 1, :5] = 7.0                                            # several units share the largest score
    desc = sf.make_desc(1, 8, 8, Hq, Hk, 8, F, nl, P, sf.SF_F32)
    gh, gf = to_dev(gh_h, "f32"), to_dev(gf_h, "f32")
    costs = ([100] * nl, [30] * nl, [7] * nl)
    dense = sum(Hq * 100 + Hk * 30 + F * 7 for _ in range(nl))
    floor = nl * (100 + 30 + 7)
    for p in range(P):
        for budget in (dense, dense // 2, dense // 3, dense // 10, floor + 4 * 7, floor + 3 * 7, floor, floor - 1):
            _budget_check(desc, gh, gf, gh_h, gf_h, p, Hk, costs, 0, budget)


# -------------------------------------------------- Sparse-MoE FFN with pruned experts (Sec. 4.5)
EPS_ROUTE = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}


def _moe_case(wl, E, top_k, forced=False, pre_ln=True, add_residual=True, sample_rows=None):
    s = wl.spec
    dtype, bf = s.dtype, ORACLE_MODE[s.dtype]
    mb = W.make_moe_block(wl, E, top_k)
    B, L, d, F, P = wl.x.shape[0], s.L, s.d, s.F, wl.P
    # keep sets of the experts: the mask kernel with "layer" = expert
    dm = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=E, P=P, dtype=SF_DTYPE[dtype], act=s.act)
    g_head = np.zeros((E, P, 8), np.float32)
    masks = sf.gate_scores_to_masks(dm, to_dev(g_head, "f32"), to_dev(mb.g_ffn, "f32"), [1] * E, mb.k_ffn.tolist())
    ref = orc.gate_scores_to_masks(g_head, mb.g_ffn, np.ones(E, np.int32), mb.k_ffn, 2)
    assert np.array_equal(to_host(masks["ffn_idx"]), ref["ffn_idx"]) and np.array_equal(to_host(masks["ffn_mask"]), ref["ffn_mask"])
    desc = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=1, P=P, dtype=SF_DTYPE[dtype], act=s.act)
    dense_dev = {k: to_dev(v, dtype) for k, v in mb.dense.items()}
    cm = sf.compact_moe_experts(desc, dense_dev, masks["ffn_idx"], top_k, mb.k_ffn.tolist())
    torch.cuda.synchronize()
    # compaction is pure data movement: bit-exact against a numpy gather
    W1c, W2Tc, b1c, b2x = to_host(cm.W1), to_host(cm.W2T), to_host(cm.b1), to_host(cm.b2x)
    for p in range(P):
        for e in range(E):
            idx = ref["ffn_idx"][e, p, :mb.k_ffn[e]]
            k = len(idx)
            assert np.array_equal(W1c[p, e, :k], mb.dense["W1"][e][idx]) and not W1c[p, e, k:].any()
            assert np.array_equal(W2Tc[p, e, :, :k], mb.dense["W2"][e][idx].T) and not W2Tc[p, e, :, k:].any()
            assert np.array_equal(b1c[p, e, :k], mb.dense["b1"][e][idx]) and not b1c[p, e, k:].any()
            assert np.array_equal(b2x[p, e], mb.dense["b2"][e])
    X = wl.x.reshape(B * L, d)
    fr = None
    if forced:
        rng = np.random.default_rng(9)
        fr = np.stack([rng.choice(E, top_k, replace=False) for _ in range(B * L)]).astype(np.int32)
    Y, route, weight, logit = sf.moe_ffn_forward(desc, cm, to_dev(X, dtype), to_dev(wl.pattern_id, dtype), pre_ln=pre_ln,
                                                 add_residual=add_residual, forced_route=to_dev(fr, dtype), want_route=True)
    Y2 = sf.moe_ffn_forward(desc, cm, to_dev(X, dtype), to_dev(wl.pattern_id, dtype), pre_ln=pre_ln,
                            add_residual=add_residual, forced_route=to_dev(fr, dtype))
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)                                # deterministic although the row order inside a segment is not
    Y, route, weight, logit = to_host(Y), to_host(route), to_host(weight), to_host(logit)
    assert np.isfinite(Y).all()
    worst, n_flip = 0.0, 0
    for p in range(P):
        rows = np.flatnonzero(np.repeat(wl.pattern_id, L) == p)
        if sample_rows is not None:                          # full-size launch: the oracle takes a sample of the rows
            rows = np.intersect1d(rows, sample_rows)
        if len(rows) == 0:
            continue
        mask = ref["ffn_mask"][:, p, :]
        y_own, r_own, w_own, lg = orc.moe_ffn(X[rows], mb.dense, top_k, act=s.act, pre_ln=pre_ln, add_residual=add_residual,
                                              bf16=bf, ffn_mask=mask, forced_route=None if fr is None else fr[rows])
        assert np.max(np.abs(logit[rows] - lg)) < (1e-4 if not bf else 3e-2)
        if fr is None:
            # margin check of the GPU's choice against the oracle's k-th largest logit
            kth = np.sort(lg, axis=1)[:, -top_k][:, None]
            eps = EPS_ROUTE[dtype] * np.maximum(1.0, np.abs(kth))
            chosen = np.zeros_like(lg, dtype=bool)
            np.put_along_axis(chosen, route[rows].astype(np.int64), True, axis=1)
            assert chosen.sum(axis=1).tolist() == [top_k] * len(rows)
            assert np.all(np.where(chosen, lg, np.inf) >= kth - eps) and np.all(np.where(~chosen, lg, -np.inf) <= kth + eps)
            n_flip += int((np.sort(route[rows], axis=1) != np.sort(r_own, axis=1)).any(axis=1).sum())
            # listed by descending logit
            lr = np.take_along_axis(logit[rows], route[rows].astype(np.int64), axis=1)
            assert np.all(np.diff(lr, axis=1) <= 0)
        else:
            assert np.array_equal(route[rows], fr[rows])
        # output reference: the oracle routed like the GPU
        y_ref, _, w_ref, _ = orc.moe_ffn(X[rows], mb.dense, top_k, act=s.act, pre_ln=pre_ln, add_residual=add_residual,
                                         bf16=bf, ffn_mask=mask, forced_route=route[rows])
        assert np.max(np.abs(weight[rows] - w_ref)) < (1e-5 if not bf else 2e-2)
        worst = max(worst, err_metric(Y[rows], y_ref))
    _say(f"   moe {s.name} E={E} k={top_k}: err {worst:.3e}, rows routed differently {n_flip}/{B * L}")
    assert worst <= TOL[dtype], worst
    assert n_flip <= max(1, (B * L if sample_rows is None else len(sample_rows)) // 100)
    return worst


@pytest.mark.parametrize("kw,E,k", [
    (dict(dtype="f32", B=3), 4, 2),
    (dict(dtype="f32", B=4, act=1, dropout="upto:2", seg=(40, 30, 50), F=96), 5, 1),
    (dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=4), 4, 2),
    (dict(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=320, seg=(100, 133, 64), extra=3, B=5, act=1, dropout="upto:2"), 8, 3),
    (dict(dtype="f32", B=2, F=64), 3, 3),                                            # every expert chosen
    (dict(dtype="f32", B=3, d=40, dh=8, F=72, seg=(20, 11, 9)), 16, 8),              # 16-expert router, widest Top-k
    (dict(dtype="bf16", d=64, dh=32, F=128, seg=(60, 40, 30), B=3), 64, 4),          # 64-expert router
])
def test_moe_ffn_parity_small(kw, E, k):
    _say(f"moe small {kw} E={E} k={k}")
    wl = make_wl(W.small_spec(**kw))
    _moe_case(wl, E, k)
    _moe_case(wl, E, k, forced=True)
    _moe_case(wl, E, k, pre_ln=False, add_residual=False)


def test_moe_ffn_parity_C2_full():
    """Full-size launch: C2's tokens (B=64, L=384, d=256, F=1024, 8 patterns) through 8 experts, Top-2."""
    _say("moe C2")
    _moe_case(make_wl(W.CONFIGS["C2"]), 8, 2)


def test_moe_ffn_parity_C5_full_sampled():
    """The launch bench.py times for the MoE block (C5's 65536 tokens, 8 experts, Top-2); the oracle computes
    768 sampled tokens (first and last rows of the batch, rows around the tile edges, random rows)."""
    _say("moe C5 sampled")
    wl = make_wl(W.CONFIGS["C5"])
    n = wl.x.shape[0] * wl.spec.L
    rng = np.random.default_rng(11)
    rows = np.unique(np.concatenate([np.arange(64), np.arange(n - 64, n), np.arange(4096 - 32, 4096 + 32),
                                     rng.choice(n, 576, replace=False)]))
    _moe_case(wl, 8, 2, sample_rows=rows)


def test_moe_forced_route_with_a_repeated_expert():
    """A caller's list that names an expert twice: the expert counts once (in its last slot), the other slot
    gets weight 0; values outside 0..E-1 are clamped.  Checked against the oracle run on the distinct experts."""
    wl = make_wl(W.small_spec(dtype="f32", B=2, dropout="none"))
    s = wl.spec
    E, k = 4, 3
    mb = W.make_moe_block(wl, E, k)
    B, L, d, F = wl.x.shape[0], s.L, s.d, s.F
    assert wl.P == 1
    desc = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=1, P=1, dtype=sf.SF_F32, act=s.act)
    ffn_idx = np.tile(np.arange(F, dtype=np.int32), (E, 1, 1))
    cm = sf.compact_moe_experts(desc, {n: to_dev(v, "f32") for n, v in mb.dense.items()}, to_dev(ffn_idx, "f32"), k, [F] * E)
    X = wl.x.reshape(B * L, d)
    fr = np.tile(np.array([[2, 0, 2]], np.int32), (B * L, 1))
    fr[1] = [7, -3, 1]                                       # clamped to [3, 0, 1]
    Y, route, weight, _ = sf.moe_ffn_forward(desc, cm, to_dev(X, "f32"), None, forced_route=to_dev(fr, "f32"), want_route=True)
    torch.cuda.synchronize()
    Y, route, weight = to_host(Y), to_host(route), to_host(weight)
    assert np.array_equal(route[0], [2, 0, 2]) and weight[0, 0] == 0.0 and np.array_equal(route[1], [3, 0, 1])
    assert np.allclose(weight.sum(axis=1), 1.0, atol=1e-6)
    y2, _, w2, _ = orc.moe_ffn(X[[0] + list(range(2, B * L))], mb.dense, 2, act=s.act, forced_route=np.tile([[0, 2]], (B * L - 1, 1)))
    assert np.max(np.abs(weight[[0] + list(range(2, B * L))][:, 1:] - w2)) < 1e-5
    assert err_metric(Y[[0] + list(range(2, B * L))], y2) <= TOL["f32"]
    y1, _, _, _ = orc.moe_ffn(X[1:2], mb.dense, 3, act=s.act, forced_route=np.array([[3, 0, 1]], np.int32))
    assert err_metric(Y[1:2], y1) <= TOL["f32"]


def test_moe_single_expert_equals_pruned_ffn():
    """E = 1, k = 1: the block is the pruned FFN of the encoder (same GEMMs, other row order; the residual
    is added after the fp32 product instead of inside the GEMM, so the last bf16 bit may differ)."""
    wl = make_wl(W.small_spec(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=3))
    s = wl.spec
    B, L, d, F, P = wl.x.shape[0], s.L, s.d, s.F, wl.P
    dmod = DeviceModel(wl).build_plan()
    ly = dmod.layers[0]
    lw = wl.layers[0]
    dense = {"Wr": np.zeros((1, d), np.float32), "br": None, "W1": lw["W1"][None], "b1": lw["b1"][None],
             "W2": lw["W2"][None], "b2": lw["b2"][None], "ln_g": lw["ln2_g"], "ln_b": lw["ln2_b"]}
    dense_dev = {k: to_dev(v, "bf16") for k, v in dense.items()}
    ffn_idx = dmod.masks["ffn_idx"][0:1].contiguous()                     # [1, P, F]
    cm = sf.compact_moe_experts(dmod.desc, dense_dev, ffn_idx, 1, [int(wl.k_ffn[0])])
    X = dmod.x.view(B * L, d)
    y_moe = sf.moe_ffn_forward(dmod.desc, cm, X, dmod.pattern_id)
    y_ffn = sf.pruned_ffn_forward(dmod.desc, ly, X, dmod.pattern_id)
    torch.cuda.synchronize()
    assert err_metric(to_host(y_moe), to_host(y_ffn)) <= 2.0 ** -7


# -------------------------------------------------- a4-a7: sparse_gqa_forward
def _gqa_case(dtype, B, nH, nG, L, dh, U_override, mask, seed, per_sample_map=False, forced=False,
              v_transposed=False, strided=False, n_sample=0):
    rng = np.random.default_rng(seed)
    q = W.storage_rounding(dtype)
    Q = q(rng.standard_normal((B, nH, L, dh)).astype(np.float32))
    K = q(rng.standard_normal((B, nG, L, dh)).astype(np.float32))
    V = q(rng.standard_normal((B, nG, L, dh)).astype(np.float32))
    n_maps = 3 if per_sample_map else 1
    hg = rng.integers(0, nG, (n_maps, nH)).astype(np.int32)
    hg[:, 0] = 0
    pid = rng.integers(0, n_maps, B).astype(np.int32) if per_sample_map else None
    kv = None
    if mask:
        kv = (rng.random((B, L)) < 0.7).astype(np.uint8)
        kv[:, L // 3: L // 3 + 40] = 0          # a whole disallowed stretch (a dropped modality)
        kv[:, 0] = 1
        if B > 1:
            kv[1] = 0
            kv[1, [1, L // 2, L - 1]] = 1        # fewer allowed queries than U
    # Hq/Hk of the descriptor describe the dense model and are not used by this entry point
    desc = sf.make_desc(B, L, 64, 8, 2, dh, 64, dtype=SF_DTYPE[dtype], U_override=U_override, n_sample=n_sample)
    U = sf.num_active(desc)
    samp = None
    if n_sample:
        # distinct keys, then a few duplicates, padding and out-of-range entries; sample 0 only hits
        # disallowed keys when a mask is on (empty intersection: every allowed query scores 0)
        samp = np.full((B, n_sample), -1, np.int32)
        for b in range(B):
            n = max(1, n_sample - 4)
            samp[b, :n] = rng.choice(L, min(n, L), replace=False)[:n]
            samp[b, n:] = [samp[b, 0], L + 3, -1, samp[b, n - 1]][: n_sample - n]
        if mask:
            bad = np.flatnonzero(kv[0] == 0)
            samp[0] = -1
            samp[0, :min(n_sample, len(bad))] = bad[:n_sample]
    hgb = hg[pid] if pid is not None else None
    fs = None
    if forced:
        fs = np.full((B, nH, U), -1, np.int32)
        for b in range(B):
            for h in range(nH):
                n = int(rng.integers(0, U + 1))
                fs[b, h, :n] = np.sort(rng.choice(L, n, replace=False))
    # device tensors (optionally as strided views of a token-major buffer, V transposed)
    if strided:
        buf = torch.zeros((B, L, (nH + 2 * nG) * dh), dtype=to_dev(Q[:1, :1, :1], dtype).dtype, device="cuda")
        buf[:, :, :nH * dh] = to_dev(Q, dtype).permute(0, 2, 1, 3).reshape(B, L, nH * dh)
        buf[:, :, nH * dh:(nH + nG) * dh] = to_dev(K, dtype).permute(0, 2, 1, 3).reshape(B, L, nG * dh)
        buf[:, :, (nH + nG) * dh:] = to_dev(V, dtype).permute(0, 2, 1, 3).reshape(B, L, nG * dh)
        Qd = buf[:, :, :nH * dh].view(B, L, nH, dh).permute(0, 2, 1, 3)
        Kd = buf[:, :, nH * dh:(nH + nG) * dh].view(B, L, nG, dh).permute(0, 2, 1, 3)
        Vd = buf[:, :, (nH + nG) * dh:].view(B, L, nG, dh).permute(0, 2, 1, 3)
    else:
        Qd, Kd, Vd = to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype)
    if v_transposed:
        Lp = (L + 7) // 8 * 8
        vt = torch.full((B, nG, dh, Lp), float("nan"), dtype=Vd.dtype, device="cuda")   # padding must not leak
        vt[..., :L] = to_dev(V, dtype).permute(0, 1, 3, 2)
        Vd = vt
    O, sel, score = sf.sparse_gqa_forward(desc, Qd, Kd, Vd, to_dev(hg, dtype), to_dev(pid, dtype),
                                          to_dev(kv, dtype), to_dev(fs, dtype), v_transposed=v_transposed,
                                          want_sel=True, want_score=True, sample_idx=to_dev(samp, dtype))
    torch.cuda.synchronize()
    O, sel, score = to_host(O), to_host(sel), to_host(score)

    bf = ORACLE_MODE[dtype]
    _, M_ref, sel_ref, _ = orc.sparse_gqa(Q, K, V, hg[0], U, kv, fs, bf, hgb, sample_idx=samp)
    n_diff = 0
    if not forced:
        for b in range(B):
            for h in range(nH):
                ok, diff = selection_report(M_ref[b, h], sel[b, h], sel_ref[b, h],
                                            None if kv is None else kv[b], EPS_SEL_OP[dtype])
                assert ok, (b, h, sel[b, h], sel_ref[b, h])
                n_diff += diff
        if U < L and U > 0:
            fin = np.isfinite(M_ref)
            assert np.array_equal(np.isneginf(score), np.isneginf(M_ref))
            assert np.max(np.abs(score[fin] - M_ref[fin]) / np.maximum(1, np.abs(M_ref[fin]))) < \
                (1e-5 if dtype == "f32" else 1e-4)
    else:
        assert np.array_equal(sel, sel_ref)
    O_ref, _, _, _ = orc.sparse_gqa(Q, K, V, hg[0], U, kv, sel, bf, hgb)
    e = err_metric(O, O_ref)
    assert np.isfinite(O).all()
    assert e <= TOL[dtype], e
    assert n_diff <= max(1, (B * nH) // 50), n_diff
    return e


@pytest.mark.parametrize("dtype,B,nH,nG,L,dh,Uo,mask", [
    ("f32", 2, 4, 2, 48, 16, -1, True),            # C1-shaped
    ("f32", 3, 3, 3, 77, 8, -1, False),            # ragged, groups = heads
    ("f32", 2, 2, 1, 130, 20, 0, True),            # U = 0: every row is the context vector
    ("f32", 2, 4, 2, 65, 12, 65, True),            # dense pattern with a key mask
    ("bf16", 2, 6, 2, 384, 32, -1, True),          # C2-shaped (dh 32)
    ("bf16", 3, 4, 4, 480, 64, -1, True),          # C3-shaped
    ("bf16", 2, 7, 2, 512, 64, -1, False),         # C4-shaped, 3+4 heads per group
    ("bf16", 1, 8, 4, 4096, 64, -1, False),        # C5-shaped: key splits
    ("bf16", 16, 9, 3, 2048, 64, -1, False),       # key splits; groups of unequal size: passes that leave waves
                                                   # without a pair, groups that need a second pass
    ("bf16", 40, 16, 8, 300, 32, -1, True),        # a (sample, group) problem per compute unit and two pairs each: the
                                                   # four-wave build of the active pass
    ("bf16", 2, 3, 1, 203, 64, -1, True),          # ragged L, one group
    ("bf16", 2, 4, 2, 333, 128, -1, True),         # dh 128
    ("bf16", 2, 4, 2, 200, 64, 200, False),        # dense pattern (U = L): flash GQA
    ("bf16", 2, 4, 2, 300, 32, 300, True),         # dense pattern with a key mask
    ("bf16", 2, 6, 2, 1024, 64, 1024, True),       # dense pattern, many tiles, 3 heads per group, key mask
    ("bf16", 1, 4, 2, 1500, 64, 1500, False),      # dense pattern, ragged last tile
    ("bf16", 2, 4, 2, 700, 32, 700, True),         # dense pattern, dh 32, key mask
    ("bf16", 1, 4, 4, 2100, 64, 333, True),        # many active rows but not all (two pairs per wave), key mask
    ("bf16", 2, 2, 2, 96, 64, 0, True),            # U = 0
    ("bf16", 1, 2, 1, 40, 64, 7, False),           # fewer rows than one MFMA block
])
def test_sparse_gqa_parity(dtype, B, nH, nG, L, dh, Uo, mask):
    _say(f"sgqa {dtype} B={B} nH={nH} nG={nG} L={L} dh={dh} U={Uo} mask={mask}")
    _gqa_case(dtype, B, nH, nG, L, dh, Uo, mask, seed=L * 7 + dh)


def test_sparse_gqa_empty_slots_with_key_splits():
    """Fewer active rows than U on a long sequence (the active pass runs in key splits and a merge kernel
    finishes the rows): the empty slots of sample 1 must not touch any row - in particular not the last row of
    sample 0, which is made an active row here so that the lazy-row fill cannot paper over a stray write."""
    B, nH, nG, L, dh = 2, 2, 1, 4096, 64
    rng = np.random.default_rng(77)
    Q = W.to_bf16_values(rng.standard_normal((B, nH, L, dh)).astype(np.float32))
    K = W.to_bf16_values(rng.standard_normal((B, nG, L, dh)).astype(np.float32))
    V = W.to_bf16_values(rng.standard_normal((B, nG, L, dh)).astype(np.float32))
    hg = np.zeros((1, nH), np.int32)
    desc = sf.make_desc(B, L, 64, 8, 2, dh, 64, dtype=sf.SF_BF16)
    U = sf.num_active(desc)
    fs = np.full((B, nH, U), -1, np.int32)
    fs[0, :, :3] = [5, 100, L - 1]
    fs[1, :, :1] = [7]
    O, sel, _ = sf.sparse_gqa_forward(desc, to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(V, "bf16"), to_dev(hg, "bf16"),
                                      None, None, to_dev(fs, "bf16"), want_sel=True)
    torch.cuda.synchronize()
    O, sel = to_host(O), to_host(sel)
    assert np.array_equal(sel, fs)
    O_ref, _, _, _ = orc.sparse_gqa(Q, K, V, hg[0], U, None, fs, True, None)
    assert np.isfinite(O).all()
    assert err_metric(O, O_ref) <= TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sparse_gqa_variants(dtype):
    dh = 16 if dtype == "f32" else 64
    _say(f"sgqa variants {dtype}")
    _gqa_case(dtype, 4, 5, 3, 150, dh, -1, True, seed=1, per_sample_map=True)
    _gqa_case(dtype, 2, 4, 2, 150, dh, -1, True, seed=2, forced=True)
    _gqa_case(dtype, 2, 4, 2, 150, dh, -1, True, seed=3, strided=True)
    _gqa_case(dtype, 2, 4, 2, 150, dh, -1, False, seed=4, v_transposed=True)
    _gqa_case(dtype, 2, 4, 2, 1150, dh, -1, True, seed=5, v_transposed=True, strided=True)


@pytest.mark.parametrize("dtype,B,nH,nG,L,dh,ns,mask", [
    ("f32", 2, 4, 2, 65, 12, 9, False), ("f32", 3, 5, 2, 300, 16, 40, True),
    ("bf16", 2, 4, 2, 300, 32, 30, True), ("bf16", 3, 6, 3, 777, 64, 35, False),
    ("bf16", 2, 8, 2, 1100, 64, 150, True), ("bf16", 2, 2, 1, 200, 128, 64, True),
])
def test_sparse_gqa_sampled_score_parity(dtype, B, nH, nG, L, dh, ns, mask):
    _say(f"sgqa sampled {dtype} B={B} nH={nH} nG={nG} L={L} dh={dh} n_sample={ns} mask={mask}")
    _gqa_case(dtype, B, nH, nG, L, dh, -1, mask, seed=L + ns)
    _gqa_case(dtype, B, nH, nG, L, dh, -1, mask, seed=L + ns, n_sample=ns)
    _gqa_case(dtype, B, nH, nG, L, dh, -1, mask, seed=L + ns + 1, n_sample=ns, per_sample_map=True, strided=True,
              v_transposed=dtype == "bf16")


def test_sparse_gqa_full_sample_equals_unsampled():
    """A sample that lists every key reproduces the unsampled operator (same kernels run on a gathered
    copy of K in the same key order)."""
    rng = np.random.default_rng(3)
    B, nH, nG, L, dh = 2, 4, 2, 384, 64
    Q, K, V = (to_dev(W.to_bf16_values(rng.standard_normal(s).astype(np.float32)), "bf16")
               for s in ((B, nH, L, dh), (B, nG, L, dh), (B, nG, L, dh)))
    hg = to_dev(np.array([[0, 0, 1, 1]], np.int32), "bf16")
    kv = (rng.random((B, L)) < 0.8).astype(np.uint8); kv[:, 0] = 1
    d0 = sf.make_desc(B, L, 64, 8, 2, dh, 64, dtype=sf.SF_BF16)
    d1 = sf.make_desc(B, L, 64, 8, 2, dh, 64, dtype=sf.SF_BF16, n_sample=L)
    full = to_dev(np.tile(np.arange(L, dtype=np.int32)[::-1], (B, 1)).copy(), "bf16")
    O0, s0, m0 = sf.sparse_gqa_forward(d0, Q, K, V, hg, None, to_dev(kv, "bf16"), want_score=True)
    O1, s1, m1 = sf.sparse_gqa_forward(d1, Q, K, V, hg, None, to_dev(kv, "bf16"), want_score=True, sample_idx=full)
    torch.cuda.synchronize()
    # the max term is identical (same MFMA products); the mean key is summed in another order, so the scores
    # agree to fp32 rounding and only an exact near-tie at the U-th score could flip a pick
    fin = torch.isfinite(m0)
    assert torch.equal(fin, torch.isfinite(m1))
    assert float((m0[fin] - m1[fin]).abs().max()) < 2e-5
    assert int((s0 != s1).sum()) <= 2
    if torch.equal(s0, s1):
        assert torch.equal(O0, O1)


def test_sparse_gqa_dense_equals_library_attention():
    """groups = heads, every row active: the kernel is plain multi-head attention."""
    torch.manual_seed(0)
    B, H, L, dh = 2, 4, 256, 64
    Q, K, V = (torch.randn(B, H, L, dh, device="cuda").to(torch.bfloat16) for _ in range(3))
    desc = sf.make_desc(B, L, 64, H, H, dh, 64, dtype=sf.SF_BF16, U_override=L)
    O, _, _ = sf.sparse_gqa_forward(desc, Q, K, V, torch.arange(H, dtype=torch.int32, device="cuda"))
    ref = torch.nn.functional.scaled_dot_product_attention(Q.cpu().double(), K.cpu().double(), V.cpu().double())
    ref = ref.permute(0, 2, 1, 3).reshape(B, L, H * dh).numpy()
    assert err_metric(to_host(O), ref) <= 2e-2


def test_sparse_gqa_is_deterministic():
    rng = np.random.default_rng(0)
    B, nH, nG, L, dh = 2, 6, 2, 1024, 64
    Q, K, V = (to_dev(W.to_bf16_values(rng.standard_normal(s).astype(np.float32)), "bf16")
               for s in ((B, nH, L, dh), (B, nG, L, dh), (B, nG, L, dh)))
    hg = torch.tensor([[0, 0, 0, 1, 1, 1]], dtype=torch.int32, device="cuda")
    desc = sf.make_desc(B, L, 64, nH, nG, dh, 64, dtype=sf.SF_BF16)
    a = sf.sparse_gqa_forward(desc, Q, K, V, hg, want_score=True)
    b = sf.sparse_gqa_forward(desc, Q, K, V, hg, want_score=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


# ------------------------------------------------------------------- a9: FFN
@pytest.mark.parametrize("dtype,act,B,L,d,F,keep", [
    ("f32", 0, 2, 48, 64, 256, 0.5), ("f32", 1, 3, 37, 40, 100, 0.33),
    ("bf16", 0, 4, 384, 256, 1024, 0.6), ("bf16", 1, 3, 203, 128, 520, 0.71), ("bf16", 0, 2, 4096, 768, 3072, 0.7),
    # 37 tile slots per XCD, four column tiles per row: rows of tiles that straddle two rounds of the persistent walk
    ("bf16", 0, 37, 512, 256, 1280, 0.8),
    # tile counts that do not divide by the XCDs or by the workgroups of an XCD, ragged row tiles
    ("bf16", 1, 23, 300, 384, 1280, 0.8), ("bf16", 0, 51, 384, 256, 1024, 0.5),
])
def test_pruned_ffn_parity(dtype, act, B, L, d, F, keep):
    _say(f"ffn {dtype} act={act} B={B} L={L} d={d} F={F}")
    _ffn_case(dtype, act, B, L, d, F, keep)


def _ffn_case(dtype, act, B, L, d, F, keep):
    spec = W.small_spec(dtype=dtype, B=B, seg=(L - 1,), extra=1, d=d, Hq=2, Hk=1, dh=32, F=F, nl=1,
                        head_keep=1.0, ffn_keep=keep, dropout="none", final_ln=False, act=act, seed=L + F)
    wl = make_wl(spec)
    # three patterns with different channel sets
    rng = np.random.default_rng(5)
    wl.pattern_bits = np.arange(3)
    wl.pattern_id = rng.integers(0, 3, B).astype(np.int32)
    wl.g_head = np.repeat(wl.g_head, 3, axis=1)
    wl.g_ffn = rng.random((1, 3, F), dtype=np.float32)
    masks = oracle_masks(wl)
    dm = DeviceModel(wl).build_plan()
    for pre_ln, res in ((True, True), (False, False)):
        Y = sf.pruned_ffn_forward(dm.desc, dm.layers[0], dm.x.view(B * L, d), dm.pattern_id, pre_ln, res)
        torch.cuda.synchronize()
        Y = to_host(Y).reshape(B, L, d)
        packs = compact_packs(wl, masks)
        for b in range(B):
            ref = orc.pruned_ffn(packs[0][wl.pattern_id[b]], wl.x[b], act=act, pre_ln=pre_ln,
                                 add_residual=res, bf16=ORACLE_MODE[dtype])
            e = err_metric(Y[b], ref)
            assert e <= TOL[dtype], (b, pre_ln, e)


# ------------------------------------------------------------ a10: encoder
def _encoder_parity(wl, samples=None, U_override=-1, max_pick_diff_frac=0.01, sample_idx=None, own_choice=True):
    s = wl.spec
    bf = ORACLE_MODE[s.dtype]
    dm = DeviceModel(wl, U_override=U_override, sample_idx=sample_idx).build_plan()
    U = sf.num_active(dm.desc)
    ref_masks = oracle_masks(wl)
    for k in MASK_KEYS:
        assert np.array_equal(to_host(dm.masks[k]), ref_masks[k]), k
    Y, sel, score = dm.forward(want_sel=True, want_score=False)
    torch.cuda.synchronize()
    Y, sel = to_host(Y), to_host(sel)
    assert np.isfinite(Y).all()
    B = wl.x.shape[0]
    samples = list(range(B)) if samples is None else samples
    packs = compact_packs(wl, ref_masks)
    kv = None if wl.key_valid is None else wl.key_valid[samples]
    # oracle with its own choice: gives the reference scores / choices for the margin check
    si = None if sample_idx is None else sample_idx[samples]
    # (reported only: how far the output moves when the oracle takes its own active sets)
    y_own = None
    if own_choice:
        y_own, _, _ = orc.encoder_forward(wl.x[samples], packs, U, wl.pattern_id[samples], kv, act=s.act,
                                          final_ln=wl.final_ln, bf16=bf, want_score=False, sample_idx=si)
    # oracle forced to the GPU's choice, layer by layer: the output reference
    y_ref, sel_chk, score_f = orc.encoder_forward(wl.x[samples], packs, U, wl.pattern_id[samples], kv, act=s.act,
                                                  forced_sel=sel[:, samples], final_ln=wl.final_ln, bf16=bf,
                                                  want_score=True, sample_idx=si)
    n_diff = n_tot = picks_diff = picks_tot = 0
    if 0 < U < s.L:
        for l in range(s.n_layers):
            for bi, b in enumerate(samples):
                for h in range(int(wl.k_head[l])):
                    # scores of the forced run are the ones this layer's GPU input corresponds to
                    m = score_f[l, bi, h]
                    ref_sel = np.sort(np.lexsort((np.arange(s.L), -m.astype(np.float32)))[:np.sum(sel[l, b, h] >= 0)])
                    ok, diff = selection_report(m, sel[l, b, h], ref_sel, None if kv is None else kv[bi],
                                                EPS_SEL_ENC[s.dtype])
                    assert ok, (l, b, h)
                    n_diff += diff
                    n_tot += 1
                    picks_diff += len(np.setdiff1d(sel[l, b, h][sel[l, b, h] >= 0], ref_sel))
                    picks_tot += len(ref_sel)
    e = err_metric(Y[samples], y_ref)
    _say(f"   encoder {s.name}: err {e:.3e}, (sample, head, layer) sets differing {n_diff}/{n_tot}, "
         f"picks differing {picks_diff}/{picks_tot}"
         + ("" if y_own is None else f", err vs oracle's own choice {err_metric(Y[samples], y_own):.3e}"))
    assert e <= TOL[s.dtype], e
    # Inside the bf16 stack Q and K carry 1-ulp rounding differences, so near-ties at the
    # U-th score may resolve differently (each such choice passed the margin check above);
    # at most 1 % of the picked queries may differ.  In fp32 the choice must be identical.
    assert picks_diff <= max(2, int(max_pick_diff_frac * picks_tot)), (picks_diff, picks_tot)
    if s.dtype == "f32":
        assert n_diff == 0
    return e


@pytest.mark.parametrize("kw", [
    dict(dtype="f32"),
    dict(dtype="f32", act=1, dropout="upto:2", B=5, c=1),
    dict(dtype="f32", dropout="none", Hq=6, Hk=3, head_keep=0.34, nl=3),
    dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=4),
    dict(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64), extra=3, B=3, nl=3,
         head_keep=(0.4, 0.9), act=1, c=3),
    # long enough that at most a quarter of the rows are active in some head: the output projection then runs on the
    # active rows only and the others take their sample's projected context vector
    dict(dtype="bf16", d=64, dh=32, Hq=4, Hk=2, F=192, seg=(250, 150, 112), B=4, c=2),
    dict(dtype="bf16", d=128, dh=32, Hq=8, Hk=4, F=256, seg=(200, 120, 130, 70), extra=2, B=5, nl=3, head_keep=(0.3, 0.6),
         act=1, c=1, dropout="upto:2"),
    dict(dtype="bf16", d=128, dh=32, Hq=4, Hk=1, F=128, seg=(300, 213), extra=0, B=2, nl=2, head_keep=0.25, c=3,
         dropout="none", final_ln=False),
])
def test_encoder_parity_small(kw):
    _say(f"encoder small {kw}")
    _encoder_parity(make_wl(W.small_spec(**kw)))


def test_encoder_parity_C1_full():
    _say("encoder C1")
    wl = make_wl(W.CONFIGS["C1"])
    _encoder_parity(wl)
    for kh in (1, 2, 3, 4):                      # the config names no head keep ratio: sweep it
        wl2 = make_wl(W.CONFIGS["C1"])
        wl2.k_head[:] = kh
        _encoder_parity(wl2)


def test_encoder_parity_C2_full():
    _say("encoder C2")
    _encoder_parity(make_wl(W.CONFIGS["C2"]))


def _spread_samples(wl, n):
    """n samples of the batch for the oracle: the first, the last, one of every presence pattern in use, the rest
    drawn (seeded) - so that a fault tied to the sample index, the tile walk or a pattern bucket is seen."""
    B = wl.x.shape[0]
    if n >= B:
        return list(range(B))
    picked = {0, B - 1, B // 2}
    for p in np.unique(wl.pattern_id):
        picked.add(int(np.flatnonzero(wl.pattern_id == p)[0]))
        picked.add(int(np.flatnonzero(wl.pattern_id == p)[-1]))
    rest = [b for b in np.random.default_rng(1).permutation(B).tolist() if b not in picked]
    return sorted(picked | set(rest[: max(0, n - len(picked))]))


@pytest.mark.parametrize("name,n_samples", [("C3", 40), ("C4", 16), ("C5", 16)])
def test_encoder_parity_full_size_sampled(name, n_samples):
    """Full-size launch (the configuration the benchmark times); the oracle recomputes whole samples, which are
    independent of the others: all 16 of C5, 16 of C4's 128, 40 of C3's 256 incl. both ends of every pattern."""
    wl = make_wl(W.CONFIGS[name])
    samples = _spread_samples(wl, n_samples)
    _say(f"encoder {name} (full batch on the GPU, {len(samples)} samples through the oracle, "
         f"{len(np.unique(wl.pattern_id[samples]))} of {wl.P} patterns)")
    assert len(np.unique(wl.pattern_id[samples])) == wl.P
    _encoder_parity(wl, samples=samples, own_choice=False)


def _key_sample(wl, n, seed):
    """n distinct keys per sample, drawn from the allowed ones (the caller's sampler is not part of the method)."""
    rng = np.random.default_rng(seed)
    B, L = wl.x.shape[0], wl.spec.L
    out = np.full((B, n), -1, np.int32)
    for b in range(B):
        allowed = np.arange(L) if wl.key_valid is None else np.flatnonzero(wl.key_valid[b])
        k = min(n, len(allowed))
        out[b, :k] = np.sort(rng.choice(allowed, k, replace=False))
    return out


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", B=3, nl=2),
    dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=4, nl=2),
    dict(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64), extra=3, B=3, nl=2, act=1),
])
def test_encoder_sampled_score_parity_small(kw):
    _say(f"encoder sampled small {kw}")
    wl = make_wl(W.small_spec(**kw))
    _encoder_parity(wl, sample_idx=_key_sample(wl, 12, 1))


@pytest.mark.parametrize("name,n_samples", [("C2", 3), ("C5", 1)])
def test_encoder_sampled_score_parity_full_size(name, n_samples):
    """Full-size launch with a key sample of U = c*ceil(ln L) keys per sample (the size that makes the
    score O(L log L))."""
    _say(f"encoder sampled {name}")
    wl = make_wl(W.CONFIGS[name])
    U = orc.num_active(wl.spec.L, wl.spec.c)
    rng = np.random.default_rng(2)
    samples = sorted(rng.choice(wl.x.shape[0], n_samples, replace=False).tolist())
    _encoder_parity(wl, samples=samples, sample_idx=_key_sample(wl, U, 3))


def test_encoder_dense_pattern_and_U0():
    _say("encoder dense pattern / U=0")
    wl = make_wl(W.small_spec(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=3))
    _encoder_parity(wl, U_override=wl.spec.L)
    _encoder_parity(wl, U_override=0)
    wl = make_wl(W.small_spec(dtype="f32", B=2))
    _encoder_parity(wl, U_override=wl.spec.L)
    _encoder_parity(wl, U_override=0)


def test_encoder_is_deterministic_and_reusable():
    wl = make_wl(W.small_spec(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90), B=4))
    dm = DeviceModel(wl).build_plan()
    y1, s1, _ = dm.forward(want_sel=True)
    y2, s2, _ = dm.forward(want_sel=True)          # same workspace, second call
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(s1, s2)


@pytest.mark.parametrize("which", ["small-bf16", "small-f32", "C2"])
def test_step_under_hip_graph_replay(which):
    """The whole step (masks + compaction + encoder) recorded into a HIP graph: every replay, with eager work
    and synchronisations in between, must reproduce the eager result bit for bit."""
    _say(f"graph replay {which}")
    if which == "C2":
        wl = make_wl(W.CONFIGS["C2"])
    else:
        wl = make_wl(W.small_spec(dtype=which.split("-")[1], d=64, dh=32, F=192, seg=(70, 50, 90), B=4, nl=2))
    dm = DeviceModel(wl).build_plan()
    y = torch.empty_like(dm.x)

    def step():
        dm.build_plan()
        dm.forward(out=y)

    step()
    torch.cuda.synchronize()
    y_eager = y.clone()
    masks_eager = {k: v.clone() for k, v in dm.masks.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        y.fill_(float("nan"))
        for v in dm.masks.values():
            v.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {rep} differs from the eager step"
        for k, v in dm.masks.items():
            assert torch.equal(v, masks_eager[k]), f"replay {rep}: {k} differs"
        step()                                     # eager work between the replays, same buffers
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager)


@pytest.mark.parametrize("which", ["small-f32", "C2"])
def test_moe_block_under_hip_graph_replay(which):
    """Expert compaction + the MoE forward (router, counting sort, grouped GEMMs, combine) recorded into a HIP
    graph: every replay, with eager work and synchronisations in between, reproduces the eager result."""
    _say(f"moe graph replay {which}")
    if which == "C2":
        wl, E, k = make_wl(W.CONFIGS["C2"]), 8, 2
    else:
        wl, E, k = make_wl(W.small_spec(dtype="f32", B=3, seg=(40, 30, 50), F=96)), 4, 2
    s = wl.spec
    dtype = s.dtype
    mb = W.make_moe_block(wl, E, k)
    B, L, d, F, P = wl.x.shape[0], s.L, s.d, s.F, wl.P
    dt = sf.SF_BF16 if dtype == "bf16" else sf.SF_F32
    dmask = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=E, P=P, dtype=dt, act=s.act)
    desc = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=1, P=P, dtype=dt, act=s.act)
    g_head = torch.zeros((E, P, 8), dtype=torch.float32, device="cuda")
    masks = sf.gate_scores_to_masks(dmask, g_head, to_dev(mb.g_ffn, "f32"), [1] * E, mb.k_ffn.tolist())
    dense = {n: to_dev(v, dtype) for n, v in mb.dense.items()}
    cm = sf.compact_moe_experts(desc, dense, masks["ffn_idx"], k, mb.k_ffn.tolist())
    X, pid = to_dev(wl.x.reshape(B * L, d), dtype), to_dev(wl.pattern_id, dtype)
    ws = sf.workspace(sf.moe_ffn_workspace_bytes(desc, cm))
    Y = torch.empty_like(X)

    def step():
        sf.compact_moe_experts(desc, dense, masks["ffn_idx"], k, mb.k_ffn.tolist(), out=cm)
        sf.moe_ffn_forward(desc, cm, X, pid, out=Y, ws=ws)

    step()
    torch.cuda.synchronize()
    y_eager = Y.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        Y.fill_(float("nan"))
        ws.zero_()
        cm.W1.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_eager), f"replay {rep} differs from the eager result"
        step()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_eager)


def test_encoder_rejects_small_workspace():
    wl = make_wl(W.small_spec(dtype="f32", B=2))
    dm = DeviceModel(wl).build_plan()
    with pytest.raises(sf.SentryFuseError, match="workspace"):
        sf.encoder_forward(dm.desc, dm.layers, dm.x, dm.pattern_id, dm.key_valid, dm.final_ln,
                           ws=torch.empty(256, dtype=torch.uint8, device="cuda"))


def test_measurement_aids_run_and_copy_is_exact():
    # the register-only MFMA loop reports its flops; the copy aid copies bit for bit (ragged tail of the 4-way unroll too)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert sf.ceiling_mfma_launch(8, 10, False, sink) == 8 * 8 * 10 * 32 * 32768
    assert sf.ceiling_mfma_launch(8, 10, True, sink) == 8 * 8 * 10 * 32 * 32768
    torch.cuda.synchronize()
    assert not sink.any()
    for n in (16, 4096 + 16, (1 << 22) + 48):
        src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
        dst = torch.zeros_like(src)
        sf.ceiling_copy_launch(src, dst)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
    with pytest.raises(sf.SentryFuseError):
        sf.ceiling_mfma_launch(0, 10, False, sink)
