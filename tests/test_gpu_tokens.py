"""GPU parity of token compaction (the tokens of absent modalities are dropped, every sample runs at its own length
with its own number of active queries) against the CPU oracle, through the C ABI.

Index work (positions, lengths, active counts, moved rows) is bit-exact.  The encoder on the compacted batch is
compared sample by sample with the oracle run on that sample's valid tokens alone (L = T_b, U = U_b, no mask): the
active-query choice under the same margin rule as the other encoder tests, the output against the oracle forced to
the GPU's choice.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as orc
from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W
from gpu_utils import DeviceModel, desc_for, selection_report, to_dev, to_host
from helpers import compact_packs, err_metric, make_wl, oracle_masks

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
EPS_SEL_ENC = {"f32": 1e-5, "bf16": 2e-2}


def _say(msg):
    print(msg, flush=True)


def _index_reference(valid, Lc, c):
    B, L = valid.shape
    slot_of = np.full((B, L), -1, np.int32)
    row_index = np.full((B, Lc), -1, np.int32)
    valid_c = np.zeros((B, Lc), np.uint8)
    length = np.zeros(B, np.int32)
    u = np.zeros(B, np.int32)
    for b in range(B):
        idx = np.nonzero(valid[b])[0]
        length[b] = len(idx)
        keep = idx[:Lc]
        slot_of[b, keep] = np.arange(len(keep))
        row_index[b, :len(keep)] = keep
        valid_c[b, :min(len(idx), Lc)] = 1
        u[b] = orc.num_active(int(len(idx)), c)              # Sec. 4.4 with T = the sample's own length
    return slot_of, row_index, valid_c, length, u


@pytest.mark.parametrize("dtype,B,L,d,Lc,c", [("f32", 7, 300, 20, 300, 5), ("bf16", 9, 1000, 64, 640, 5),
                                              ("bf16", 4, 257, 8, 100, 3), ("f32", 3, 5000, 6, 5000, 5)])
def test_token_compact_indices_and_rows(dtype, B, L, d, Lc, c):
    _say(f"token compact {dtype} B={B} L={L} Lc={Lc}")
    rng = np.random.default_rng(L + B)
    valid = (rng.random((B, L)) < rng.uniform(0.1, 0.9, (B, 1))).astype(np.uint8)
    valid[0] = 1                                             # nothing dropped
    valid[1] = 0                                             # nothing left
    valid[2] = 0; valid[2, L - 1] = 1                        # one token, the last
    x = rng.standard_normal((B, L, d)).astype(np.float32)
    if dtype == "bf16":
        x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    desc = sf.make_desc(B, L, d, 1, 1, 8, 8, dtype=sf.SF_BF16 if dtype == "bf16" else sf.SF_F32, c_factor=c)
    out = sf.token_compact(desc, to_dev(x, dtype), to_dev(valid, dtype), Lc)
    torch.cuda.synchronize()
    slot_of, row_index, valid_c, length, u = _index_reference(valid, Lc, c)
    assert np.array_equal(to_host(out["len"]), length)
    assert np.array_equal(to_host(out["u_active"]), u)
    assert np.array_equal(to_host(out["slot_of"]), slot_of)
    assert np.array_equal(to_host(out["row_index"]), row_index)
    assert np.array_equal(to_host(out["valid_c"]), valid_c)
    xc = np.zeros((B, Lc, d), np.float32)
    for b in range(B):
        n = int((row_index[b] >= 0).sum())
        xc[b, :n] = x[b, row_index[b, :n]]
    assert np.array_equal(to_host(out["Xc"]), xc)
    # back: kept tokens return to their places, dropped tokens (and those lost to a small Lc) are zero rows
    back = to_host(sf.token_scatter(desc, out["Xc"], out["slot_of"]))
    assert np.array_equal(back, x * (slot_of >= 0)[:, :, None])


def _ragged_case(wl, samples=None):
    s = wl.spec
    bf = s.dtype == "bf16"
    assert wl.key_valid is not None
    dm = DeviceModel(wl).build_plan()
    ref_masks = oracle_masks(wl)
    packs = compact_packs(wl, ref_masks)
    B = wl.x.shape[0]
    lens = wl.key_valid.sum(axis=1).astype(int)
    assert len(np.unique(lens)) > 1 and lens.min() < s.L        # the case really is ragged
    Lc = int(-(-lens.max() // 8) * 8)                         # the caller knows the patterns, hence the lengths
    Lc = min(Lc, s.L)
    u_host = np.array([orc.num_active(int(t), s.c) for t in lens])
    Umax = int(u_host.max())
    tc = sf.token_compact(dm.desc, dm.x, dm.key_valid, Lc)
    dc = desc_for(wl, U_override=Umax)
    dc.L = Lc
    Yc, sel, _ = sf.encoder_forward_ragged(dc, dm.layers, tc["Xc"], dm.pattern_id, tc["valid_c"], tc["u_active"],
                                           final_ln=dm.final_ln, want_sel=True)
    Y = sf.token_scatter(dm.desc, Yc, tc["slot_of"])
    torch.cuda.synchronize()
    assert np.array_equal(to_host(tc["len"]), lens) and np.array_equal(to_host(tc["u_active"]), u_host)
    Yc, sel, Y = to_host(Yc), to_host(sel), to_host(Y)
    worst, picks_diff, picks_tot = 0.0, 0, 0
    for b in (range(B) if samples is None else samples):
        T, Ub = int(lens[b]), int(u_host[b])
        keep = np.nonzero(wl.key_valid[b])[0]
        xb = wl.x[b, keep][None]
        pid = wl.pattern_id[[b]]
        assert (sel[:, b, :, Ub:] == -1).all()
        fs = np.ascontiguousarray(sel[:, [b], :, :Ub])
        y_ref, _, score_f = orc.encoder_forward(xb, packs, Ub, pid, None, act=s.act, forced_sel=fs, final_ln=wl.final_ln,
                                                bf16=bf, want_score=True)
        if 0 < Ub < T:
            for l in range(s.n_layers):
                for h in range(int(wl.k_head[l])):
                    m = score_f[l, 0, h]
                    ref_sel = np.sort(np.lexsort((np.arange(T), -m.astype(np.float32)))[:Ub])
                    ok, diff = selection_report(m, sel[l, b, h, :Ub], ref_sel, None, EPS_SEL_ENC[s.dtype])
                    assert ok, (l, b, h)
                    picks_diff += len(np.setdiff1d(sel[l, b, h, :Ub], ref_sel))
                    picks_tot += Ub
        worst = max(worst, err_metric(Yc[b, :T], y_ref[0]))
        # full-length output: the sample's rows at their original places, zero rows for the dropped tokens
        assert np.array_equal(Y[b, keep], Yc[b, :T])
        gone = np.setdiff1d(np.arange(s.L), keep)
        assert not Y[b, gone].any()
    _say(f"   ragged encoder {s.name}: lens {lens.min()}..{lens.max()} (L {s.L}, Lc {Lc}), U_b {u_host.min()}..{Umax}, "
         f"err {worst:.3e}, picks differing {picks_diff}/{picks_tot}")
    assert worst <= TOL[s.dtype], worst
    assert picks_diff <= max(2, int(0.03 * picks_tot)), (picks_diff, picks_tot)
    if s.dtype == "f32":
        assert picks_diff == 0
    return worst


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", dropout="upto:2", B=5),
    dict(dtype="f32", dropout="upto:2", B=4, nl=2, act=1, c=2),
    dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90, 40), B=6, dropout="upto:2"),
    dict(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64, 120), B=5, nl=2, dropout="upto:3", act=1),
    # long enough for the output projection to run on the active rows only, with per-sample active counts
    dict(dtype="bf16", d=64, dh=32, Hq=4, Hk=2, F=192, seg=(260, 140, 120, 60), B=6, nl=2, dropout="upto:2", c=1),
])
def test_encoder_ragged_parity_small(kw):
    _say(f"ragged encoder {kw}")
    _ragged_case(make_wl(W.small_spec(**kw)))


def test_encoder_ragged_parity_C3_samples():
    """The dropout workload at full size (4 modalities of 256/128/64/32 tokens, up to two dropped): every sample at
    its own length in the launch configuration the benchmark times; the oracle on 6 samples of different lengths."""
    _say("ragged encoder C3")
    wl = make_wl(W.CONFIGS["C3"])
    lens = wl.key_valid.sum(axis=1)
    pick = []
    for t in np.unique(lens):
        pick.append(int(np.nonzero(lens == t)[0][0]))
    _ragged_case(wl, samples=pick[:6])


def test_ragged_entry_rejects_what_it_cannot_run():
    wl = make_wl(W.small_spec(dtype="f32", dropout="upto:2", B=3))
    dm = DeviceModel(wl).build_plan()
    tc = sf.token_compact(dm.desc, dm.x, dm.key_valid, wl.spec.L)
    dc = desc_for(wl, U_override=wl.spec.L)                 # U >= L: every row active, no per-sample counts
    with pytest.raises(sf.SentryFuseError):
        sf.encoder_forward_ragged(dc, dm.layers, tc["Xc"], dm.pattern_id, tc["valid_c"], tc["u_active"],
                                  final_ln=dm.final_ln)
    with pytest.raises(sf.SentryFuseError):
        sf.token_compact(dm.desc, dm.x, dm.key_valid, wl.spec.L + 1)


def test_compact_encode_scatter_under_hip_graph_replay():
    """Compaction, the ragged encoder and the scatter recorded into one HIP graph: every replay, with eager work and
    synchronisations in between, reproduces the eager result (no step of the chain needs the host)."""
    _say("token compaction graph replay")
    wl = make_wl(W.small_spec(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90, 40), B=6, dropout="upto:2"))
    s = wl.spec
    dm = DeviceModel(wl).build_plan()
    lens = wl.key_valid.sum(axis=1).astype(int)
    Lc = min(int(-(-lens.max() // 8) * 8), s.L)
    dc = desc_for(wl, U_override=max(orc.num_active(int(t), s.c) for t in lens))
    dc.L = Lc
    ws = sf.workspace(sf.encoder_workspace_bytes(dc, dm.layers))

    def chain():
        tc = sf.token_compact(dm.desc, dm.x, dm.key_valid, Lc)
        Yc, _, _ = sf.encoder_forward_ragged(dc, dm.layers, tc["Xc"], dm.pattern_id, tc["valid_c"], tc["u_active"],
                                             final_ln=dm.final_ln, ws=ws)
        return sf.token_scatter(dm.desc, Yc, tc["slot_of"])

    y_eager = chain().clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        y_graph = chain()
    torch.cuda.synchronize()
    for rep in range(4):
        y_graph.fill_(float("nan"))
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {rep} differs from the eager result"
        assert torch.equal(chain(), y_eager)
        torch.cuda.synchronize()
