"""GPU parity of the encoder with the attention projections in FP8 arithmetic (E4M3 codes on both operands of the
Q/K/V and of the output projection), alone and together with FP8 FFNs, against the CPU oracle, through the C ABI.

A code is a floating-point decision, so the stack is walked decision by decision: the compacted code buffers
bit-exact; the active queries by the margin rule on the oracle's scores of the device's earlier decisions; the codes
of LN1(x) and of the attention output of layer l against the oracle's own on the device's decisions before them
(equal up to one grid step plus the bf16 path's rounding noise, and equal in all but a small fraction); the output
against the oracle run on all of the device's decisions, max |a-b| / max(1,|b|) <= 2e-2.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as orc
from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W
from gpu_utils import ORACLE_MODE, DeviceModel, selection_report, to_dev, to_host
from helpers import dense_packs, err_metric, make_wl, oracle_masks

pytestmark = pytest.mark.gpu

DEC = np.array([orc.fp8_e4m3_decode(i) if (i & 0x7F) != 0x7F else 0.0 for i in range(256)])
SX1, SA = 8.0 / 448, 4.0 / 448


def _say(msg):
    print(msg, flush=True)


def _cast_e4m3(a):
    """PyTorch's cast as the offline weight quantiser (inputs inside +-448)."""
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def _build(kw, with_ffn8):
    wl = make_wl(kw if isinstance(kw, W.Spec) else W.small_spec(**kw))
    s = wl.spec
    dm = DeviceModel(wl).build_plan()
    masks = oracle_masks(wl)
    p8, cps, f8, cfs = [], [], [], []
    for l in range(s.n_layers):
        lw = wl.layers[l]
        s_qkv = float(np.float32(max(np.abs(lw[k]).max() for k in ("Wq", "Wk", "Wv")) / 448))
        so = float(np.float32(np.abs(lw["Wo"]).max() / 448))
        c8 = {k: _cast_e4m3(lw[k] / np.float32(s_qkv if k != "Wo" else so)) for k in ("Wq", "Wk", "Wv", "Wo")}
        p8.append(dict(Wq8=c8["Wq"], Wk8=c8["Wk"], Wv8=c8["Wv"], Wo8=c8["Wo"], s_qkv=s_qkv, so=so, sx1=SX1, sa=SA))
        d8 = {k: to_dev(v, "bf16") for k, v in c8.items()}
        cps.append(sf.compact_proj_fp8(dm.desc, l, d8, s_qkv, so, dm.masks, int(wl.k_head[l]), SX1, SA))
        if with_ffn8:
            s1, s2 = float(np.float32(np.abs(lw["W1"]).max() / 448)), float(np.float32(np.abs(lw["W2"]).max() / 448))
            W1q, W2q = _cast_e4m3(lw["W1"] / np.float32(s1)), _cast_e4m3(lw["W2"] / np.float32(s2))
            f8.append(dict(W1q=W1q, W2q=W2q, s1=s1, s2=s2, sx=4.0 / 448, sh=4.0 / 448))
            e8 = dict(dm.dense[l], W1=to_dev(W1q, "bf16"), W2=to_dev(W2q, "bf16"))
            cfs.append(sf.compact_ffn_fp8(dm.desc, l, e8, dict(W1=s1, W2=s2), dm.masks, int(wl.k_ffn[l]), 4.0 / 448,
                                          4.0 / 448))
    return wl, dm, masks, p8, cps, (f8 if with_ffn8 else None), (cfs if with_ffn8 else None)


def _compacted_ok(wl, masks, p8, cps):
    """the compact code buffers are the kept rows of the dense codes, bit for bit"""
    s = wl.spec
    for l, (pj, cp) in enumerate(zip(p8, cps)):
        kh = int(wl.k_head[l])
        Wqkv8, WoT8 = to_host(cp.Wqkv8), to_host(cp.WoT8)
        for p in range(Wqkv8.shape[0]):
            hi = masks["head_idx"][l, p, :kh]
            ng = int(masks["n_groups"][l, p])
            gi = masks["group_idx"][l, p, :ng]
            rows = lambda idx: (np.asarray(idx)[:, None] * s.dh + np.arange(s.dh)[None, :]).reshape(-1)
            want = np.zeros_like(Wqkv8[p])
            want[:kh * s.dh] = pj["Wq8"][rows(hi)]
            want[kh * s.dh:kh * s.dh + ng * s.dh] = pj["Wk8"][rows(gi)]
            want[(kh + s.Hk) * s.dh:(kh + s.Hk) * s.dh + ng * s.dh] = pj["Wv8"][rows(gi)]
            assert np.array_equal(Wqkv8[p], want), (l, p)
            assert np.array_equal(WoT8[p][:, :kh * s.dh], pj["Wo8"][rows(hi)].T), (l, p)
            assert not WoT8[p][:, kh * s.dh:].any()


def _case(kw, with_ffn8, samples=None):
    """samples: the samples the oracle recomputes (all by default); the device always runs the whole batch"""
    wl, dm, masks, p8, cps, f8, cfs = _build(kw, with_ffn8)
    s = wl.spec
    _compacted_ok(wl, masks, p8, cps)
    packs = dense_packs(wl, masks)
    U = sf.num_active(dm.desc)
    L, d, F, nl, dh = s.L, s.d, s.F, s.n_layers, s.dh
    Bd = wl.x.shape[0]
    samples = list(range(Bd)) if samples is None else samples
    B = len(samples)
    x_s, pid_s = wl.x[samples], wl.pattern_id[samples]
    kv_s = None if wl.key_valid is None else wl.key_valid[samples]
    Y, sel, codes = sf.encoder_forward_fp8(dm.desc, dm.layers, dm.x, ffn8=cfs, proj8=cps, pattern_id=dm.pattern_id,
                                           key_valid=dm.key_valid, final_ln=dm.final_ln, want_sel=True, want_codes=True)
    torch.cuda.synchronize()
    Y, sel = to_host(Y), to_host(sel)
    assert np.isfinite(Y).all()
    Y, sel = Y[samples], sel[:, samples]
    aq = to_host(codes["aq"]).reshape(nl, Bd, L, d)[:, samples]
    # the device's decisions in the dense head / channel layout of each sample's pattern
    oq = np.zeros((nl, B, L, s.Hq * dh), np.uint8)
    sel_dense = np.full((nl, B, s.Hq, U), -1, np.int32)
    hq = np.zeros((nl, B, L, F), np.uint8)
    for l in range(nl):
        kh, kf = int(wl.k_head[l]), int(wl.k_ffn[l])
        o = to_host(codes["oq"][l]).reshape(Bd, L, -1)[samples]
        assert not o[:, :, kh * dh:].any()                              # padding columns: code 0
        o = o[:, :, :kh * dh].reshape(B, L, kh, dh)
        for b in range(B):
            p = int(pid_s[b])
            hi = masks["head_idx"][l, p, :kh]
            oq[l, b].reshape(L, s.Hq, dh)[:, hi] = o[b]
            sel_dense[l, b, hi] = sel[l, b, :kh]
            if with_ffn8:
                h = to_host(codes["hq"][l]).reshape(Bd, L, -1)[samples]
                hq[l, b][:, masks["ffn_idx"][l, p, :kf]] = h[b, :, :kf]
    common = dict(act=s.act, final_ln=wl.final_ln, bf16=ORACLE_MODE[s.dtype], proj8=p8, forced_sel=sel_dense)
    forced = dict(aq_forced=aq, oq_forced=oq)
    if with_ffn8:
        common["ffn8"] = f8
        forced.update(xq_forced=to_host(codes["xq"]).reshape(nl, Bd, L, d)[:, samples], hq_forced=hq)
    # the oracle on all of the device's decisions: the output reference, and the scores its choices are judged on
    _say("   oracle: output reference on the device's decisions")
    y_ref, _, score_f = orc.encoder_forward(x_s, packs, U, pid_s, kv_s, want_score=True, **forced,
                                            **common)
    e = err_metric(Y, y_ref)
    picks_diff = picks_tot = 0
    if 0 < U < L:
        for l in range(nl):
            for b in range(B):
                for h in masks["head_idx"][l, int(pid_s[b]), :int(wl.k_head[l])]:
                    m = score_f[l, b, h]
                    got = sel_dense[l, b, h]
                    ref_sel = np.sort(np.lexsort((np.arange(L), -m.astype(np.float32)))[:np.sum(got >= 0)])
                    ok, _ = selection_report(m, got, ref_sel, None if kv_s is None else kv_s[b], 2e-2)
                    assert ok, (l, b, h)
                    picks_diff += len(np.setdiff1d(got[got >= 0], ref_sel))
                    picks_tot += len(ref_sel)
        assert picks_diff <= max(2, int(0.03 * picks_tot)), (picks_diff, picks_tot)
    # the codes, layer by layer: the oracle's own of layer l on the device's decisions before them
    # (deep stacks: the first and the last layer - the walk costs two oracle runs per layer - the others keep the
    # device's codes, which the output comparison above and the last layer's own codes depend on)
    aq_own, oq_own = aq.copy(), oq.copy()
    for l in (range(nl) if nl <= 3 else (0, nl - 1)):
        _say(f"   oracle: own codes of layer {l} on the device's earlier decisions")
        kw_l = dict(want_codes=True, **forced, **common)
        if with_ffn8:
            kw_l.update(n_forced_x=l, n_forced_h=l)
        r = orc.encoder_forward(x_s, packs, U, pid_s, kv_s, n_forced_a=l, n_forced_o=l, **kw_l)
        aq_own[l] = r[5][l]
        r = orc.encoder_forward(x_s, packs, U, pid_s, kv_s, n_forced_a=l + 1, n_forced_o=l, **kw_l)
        oq_own[l] = r[6][l]
    va_d, va_o = DEC[aq] * SX1, DEC[aq_own] * SX1
    bad = np.argwhere(np.abs(va_d - va_o) > 2.0 ** -3 * np.abs(va_o) + 2e-2 * np.maximum(1.0, np.abs(va_o)))
    assert len(bad) == 0, f"{len(bad)} LN1 codes off, first (layer, sample, row, column): {bad[:8].tolist()}"
    vo_d, vo_o = DEC[oq] * SA, DEC[oq_own] * SA
    bad = np.argwhere(np.abs(vo_d - vo_o) > 2.0 ** -3 * np.abs(vo_o) + 2e-2 * np.maximum(1.0, np.abs(vo_o)))
    assert len(bad) == 0, (f"{len(bad)} attention-output codes off, first (layer, sample, row, column): {bad[:8].tolist()}, "
                           f"rows {np.unique(bad[:, 2])[:16].tolist()}")
    same_a, same_o = float((aq == aq_own).mean()), float((oq == oq_own).mean())
    _say(f"   encoder with fp8 projections{' and fp8 ffn' if with_ffn8 else ''}: err {e:.3e}; LN1 codes equal to the "
         f"oracle's own {same_a:.4f}, attention-output codes {same_o:.4f}; picks differing {picks_diff}/{picks_tot}")
    assert same_a >= 0.97 and same_o >= 0.97
    assert e <= 2e-2, e


@pytest.mark.parametrize("kw,with_ffn8", [
    (dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(100, 60, 70), extra=2, B=3, nl=2, head_keep=0.5,
          ffn_keep=0.6, dropout="bernoulli:0.3"), False),
    (dict(dtype="bf16", d=384, dh=32, Hq=12, Hk=4, F=640, seg=(128, 128), extra=0, B=2, nl=1, head_keep=0.67,
          ffn_keep=0.8, act=1, dropout="none", final_ln=False), False),
    (dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(260, 140, 120), extra=2, B=2, nl=2, head_keep=0.5,
          ffn_keep=0.6, dropout="bernoulli:0.3"), True),
    # 3 kept heads of 64: 192 attention-output features, code rows padded to 256
    (dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(100, 60, 70), extra=2, B=3, nl=2, head_keep=0.75,
          ffn_keep=0.6, dropout="bernoulli:0.3"), False),
    (dict(dtype="bf16", d=256, dh=32, Hq=8, Hk=2, F=512, seg=(600, 300, 200), extra=0, B=2, nl=1, head_keep=0.6, c=4,
          ffn_keep=0.6, dropout="upto:1", final_ln=False), True),
    # long enough for the output projection to run on the active rows only (256 compact rows per sample): codes of
    # the compact rows, FP8 GEMM on them, the lazy rows' shared vector from the codes of the context vector
    (dict(dtype="bf16", d=256, dh=32, Hq=8, Hk=2, F=512, seg=(600, 300, 200), extra=0, B=2, nl=2, head_keep=0.5, c=5,
          ffn_keep=0.6, dropout="bernoulli:0.3"), True),
    (dict(dtype="bf16", d=256, dh=32, Hq=8, Hk=2, F=512, seg=(600, 300, 200), extra=0, B=2, nl=1, head_keep=0.5, c=5,
          ffn_keep=0.6, dropout="none", final_ln=False), False),
])
def test_encoder_with_fp8_projections_parity(kw, with_ffn8):
    _say(f"encoder fp8 projections {kw} ffn8={with_ffn8}")
    _case(kw, with_ffn8)


def test_encoder_fp8_C5_full_size_sampled():
    """The launch bench.py times for this path (C5, projections and FFN in FP8 arithmetic, active-row output
    projection); the oracle recomputes the first and the last sample, which are independent of the others."""
    _say("encoder fp8 projections + ffn, C5 (full batch on the GPU, 2 samples through the oracle)")
    _case(W.CONFIGS["C5"], True, samples=[0, 15])


@pytest.mark.parametrize("name,samples", [("C3", [0, 5, 77, 255]), ("C4", [0, 127])])
def test_encoder_fp8_other_configs_full_size_sampled(name, samples):
    """The other single-GPU configurations at full size: many presence patterns (C3); six layers with kept-head
    counts whose code rows need padding, and a final LayerNorm (C4)."""
    _say(f"encoder fp8 projections + ffn, {name} (full batch on the GPU, samples {samples} through the oracle)")
    _case(W.CONFIGS[name], True, samples=samples)


def test_encoder_fp8_projections_rejects_what_it_cannot_run():
    kw = dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(100, 60, 70), extra=2, B=2, nl=1, head_keep=0.5,
              ffn_keep=0.6, dropout="none")
    wl, dm, masks, p8, cps, _, _ = _build(kw, False)
    # the plain encoder's workspace is too small for this path
    small = sf.workspace(sf.encoder_workspace_bytes(dm.desc, dm.layers), dm.x.device)
    big = sf.encoder_fp8_workspace_bytes(dm.desc, dm.layers)
    if small.numel() < big:
        with pytest.raises(sf.SentryFuseError):
            sf.encoder_forward_fp8(dm.desc, dm.layers, dm.x, proj8=cps, pattern_id=dm.pattern_id, key_valid=dm.key_valid,
                                   final_ln=dm.final_ln, ws=small)
    with pytest.raises(sf.SentryFuseError):                  # neither part in FP8
        sf.encoder_forward_fp8(dm.desc, dm.layers, dm.x, pattern_id=dm.pattern_id, key_valid=dm.key_valid,
                               final_ln=dm.final_ln)
    cps[0].struct.k_head = 3                                 # not the compact layer's
    with pytest.raises(sf.SentryFuseError):
        sf.encoder_forward_fp8(dm.desc, dm.layers, dm.x, proj8=cps, pattern_id=dm.pattern_id, key_valid=dm.key_valid,
                               final_ln=dm.final_ln)
    cps[0].struct.k_head = 2
    cps[0].struct.sa = 0.0
    with pytest.raises(sf.SentryFuseError):
        sf.encoder_forward_fp8(dm.desc, dm.layers, dm.x, proj8=cps, pattern_id=dm.pattern_id, key_valid=dm.key_valid,
                               final_ln=dm.final_ln)
    # Wq, Wk, Wv with different scales cannot form one operand
    d8 = {k: to_dev(p8[0][k + "8"], "bf16") for k in ("Wq", "Wk", "Wv", "Wo")}
    nul = sf.C.c_void_p(None)
    ds = sf.SfDenseLayerFp8(sf._ptr(d8["Wq"]), sf._ptr(d8["Wk"]), sf._ptr(d8["Wv"]), sf._ptr(d8["Wo"]), nul, nul,
                            0.5, 0.25, 0.5, 0.5, 0.0, 0.0, *([nul] * 10))
    rc = sf.lib().sf_compact_proj_fp8(sf.C.byref(dm.desc), 0, sf.C.byref(ds), sf._ptr(dm.masks["head_idx"]),
                                      sf._ptr(dm.masks["group_idx"]), sf._ptr(dm.masks["n_groups"]),
                                      sf.C.byref(cps[0].struct), None)
    assert rc != 0


def test_encoder_fp8_under_hip_graph_replay():
    """The encoder with projections and FFNs in FP8 arithmetic (active-row output projection included) recorded into
    a HIP graph: every replay, with eager work and synchronisations in between, reproduces the eager result bit for
    bit."""
    _say("encoder fp8 graph replay")
    kw = dict(dtype="bf16", d=256, dh=32, Hq=8, Hk=2, F=512, seg=(600, 300, 200), extra=0, B=2, nl=2, head_keep=0.5,
              c=5, ffn_keep=0.6, dropout="bernoulli:0.3")
    wl, dm, masks, p8, cps, f8, cfs = _build(kw, True)
    ws = sf.workspace(sf.encoder_fp8_workspace_bytes(dm.desc, dm.layers), dm.x.device)
    out = torch.empty_like(dm.x)

    def run():
        sf.encoder_forward_fp8(dm.desc, dm.layers, dm.x, ffn8=cfs, proj8=cps, pattern_id=dm.pattern_id,
                               key_valid=dm.key_valid, final_ln=dm.final_ln, out=out, ws=ws)

    run()
    torch.cuda.synchronize()
    y_eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    torch.cuda.synchronize()
    for rep in range(4):
        out.fill_(float("nan"))
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, y_eager), f"replay {rep} differs from the eager result"
        run()
        torch.cuda.synchronize()
        assert torch.equal(out, y_eager)
