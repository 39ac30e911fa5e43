"""GPU parity of token compaction without padding (the valid tokens of all samples back to back, samples ordered by
presence pattern, every pattern's run of rows starting on a multiple of 256) against the CPU oracle, through the C ABI.

Index work (lengths, active counts, first rows, row maps, block patterns, moved rows) is bit-exact against a layout
written out in numpy and against the properties that define it.  The encoder over the packed rows is compared
sample by sample with the oracle run on that sample's valid tokens alone (L = T_b, U = U_b, no mask): the
active-query choice under the margin rule of the other encoder tests, the output against the oracle forced to the
GPU's choice - the bar of the padded form (tests/test_gpu_tokens.py), whose output the packed form is also held
against.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as orc
from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W
from gpu_utils import ORACLE_MODE, DeviceModel, desc_for, selection_report, to_dev, to_host
from helpers import compact_packs, err_metric, make_wl, oracle_masks

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
EPS_SEL_ENC = {"f32": 1e-5, "bf16": 2e-2}


def _say(msg):
    print(msg, flush=True)


def _up(n, m):
    return -(-int(n) // m) * m


def _layout_reference(valid, pattern, P, Tc, c):
    """The packed layout written out: runs by pattern (ascending), samples by number inside a run, runs padded to 256
    rows, align(L, 256) rows of slack with the last run's pattern; the empty plan when the rows do not fit."""
    B, L = valid.shape
    lens = valid.sum(axis=1).astype(np.int32)
    row0, ext = np.zeros(B, np.int32), np.zeros(B, np.int32)
    blk = np.full(Tc // 256, -1, np.int32)
    base, tail = 0, None
    for p in range(P):
        members = [b for b in range(B) if pattern[b] == p]
        seg0 = base
        for b in members:
            row0[b], ext[b] = base, lens[b]
            base += int(lens[b])
        if base > seg0:
            end = _up(base, 256)
            ext[members[-1]] = end - row0[members[-1]]
            blk[seg0 // 256:min(end // 256, len(blk))] = p
            base, tail = end, (members[-1], p)
    need = base + _up(L, 256) if base else 0
    fits = need <= Tc
    if fits and base:
        blk[base // 256:need // 256] = tail[1]
        ext[tail[0]] += _up(L, 256)
    if not fits:
        row0[:], ext[:], blk[:] = 0, 0, -1
    src = np.full(Tc, -1, np.int32)
    dst = np.full((B, L), -1, np.int32)
    valid_c = np.zeros((B, L), np.uint8)
    u = np.zeros(B, np.int32)
    if fits and base:
        for b in range(B):
            idx = np.nonzero(valid[b])[0]
            src[row0[b]:row0[b] + len(idx)] = b * L + idx
            dst[b, idx] = row0[b] + np.arange(len(idx))
            valid_c[b, :len(idx)] = 1
            u[b] = orc.num_active(int(len(idx)), c)              # Sec. 4.4 with T = the sample's own length
    return dict(len=lens, u_active=u, row0=row0, ext=ext, valid_c=valid_c, blk_pattern=blk, src_row=src, dst_row=dst,
                n_rows=np.array([need if fits else 0, need], np.int32))


def _check_layout_properties(valid, pattern, plan_host, Tc):
    """What the layout has to guarantee, stated without the construction."""
    B, L = valid.shape
    src, dst, blk, row0, ext = (plan_host[k] for k in ("src_row", "dst_row", "blk_pattern", "row0", "ext"))
    lens = valid.sum(axis=1).astype(np.int64)
    row0, ext = row0.astype(np.int64), ext.astype(np.int64)
    used = int(plan_host["n_rows"][0])
    # every valid token has exactly one packed row and the two maps are inverse to each other
    tok = np.nonzero(valid.reshape(-1))[0]
    assert np.array_equal(np.sort(src[src >= 0]), tok)
    assert np.array_equal(dst.reshape(-1)[src[src >= 0]], np.nonzero(src >= 0)[0])
    assert ((dst >= 0) == (valid != 0)).all()
    for b in range(B):
        rows = dst[b][valid[b] != 0]
        assert np.array_equal(rows, row0[b] + np.arange(lens[b]))      # contiguous, in token order
        assert row0[b] + L <= used or lens[b] == 0                     # L rows can be read from its first row
        if lens[b]:
            assert (blk[row0[b] // 256:(row0[b] + lens[b] - 1) // 256 + 1] == pattern[b]).all()
    # the rows the samples answer for tile the rows in use: no row of a used block is left undefined
    owners = sorted((int(row0[b]), int(ext[b])) for b in range(B) if ext[b] > 0)
    pos = 0
    for r, e in owners:
        assert r == pos
        pos += e
    assert pos == used
    assert (blk[:used // 256] >= 0).all() and (blk[used // 256:] == -1).all() and used % 256 == 0
    # runs in pattern order
    pat_rows = blk[:used // 256]
    body = pat_rows[:len(pat_rows) - _up(L, 256) // 256] if used else pat_rows
    assert (np.diff(body) >= 0).all()


@pytest.mark.parametrize("dtype,B,L,d,P,c,tight", [("f32", 7, 300, 20, 3, 5, False), ("bf16", 40, 480, 64, 11, 5, True),
                                                   ("bf16", 5, 257, 8, 1, 3, False), ("f32", 3, 5000, 8, 4, 5, True),
                                                   ("bf16", 1100, 96, 16, 6, 5, True), ("bf16", 700, 40, 16, 300, 5, True)])
def test_token_pack_layout_and_rows(dtype, B, L, d, P, c, tight):
    _say(f"token pack {dtype} B={B} L={L} P={P} tight={tight}")
    rng = np.random.default_rng(L + B)
    valid = (rng.random((B, L)) < rng.uniform(0.1, 0.9, (B, 1))).astype(np.uint8)
    valid[0] = 1                                             # nothing dropped
    valid[1] = 0                                             # nothing left
    valid[2] = 0; valid[2, L - 1] = 1                        # one token, the last
    pattern = rng.integers(0, P, B).astype(np.int32)
    if P > 2:
        pattern[pattern == 1] = 0                            # a pattern without samples
        pattern[1] = 2                                       # the empty sample is the last of its pattern or not
    x = rng.standard_normal((B, L, d)).astype(np.float32)
    if dtype == "bf16":
        x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    desc = sf.make_desc(B, L, d, 1, 1, 8, 8, dtype=sf.SF_BF16 if dtype == "bf16" else sf.SF_F32, c_factor=c, P=P)
    Tmax = sf.token_pack_rows_max(desc)
    ref_any = _layout_reference(valid, pattern, P, Tmax, c)
    Tc = int(ref_any["n_rows"][1]) if tight else Tmax
    assert Tc <= Tmax
    ref = _layout_reference(valid, pattern, P, Tc, c)
    pid = to_dev(pattern, dtype) if P > 1 else None
    Xp, plan = sf.token_pack(desc, to_dev(x, dtype), to_dev(valid, dtype), pid, Tc=Tc)
    torch.cuda.synchronize()
    got = {k: to_host(getattr(plan, k)) for k in ref}
    for k in ref:
        assert np.array_equal(got[k], ref[k]), k
    _check_layout_properties(valid, pattern, got, Tc)
    xp = np.zeros((Tc, d), np.float32)
    rows = ref["src_row"] >= 0
    xp[rows] = x.reshape(B * L, d)[ref["src_row"][rows]]
    assert np.array_equal(to_host(Xp), xp)
    back = to_host(sf.token_unpack(desc, Xp, plan))
    assert np.array_equal(back, x * (valid != 0)[:, :, None])
    # a buffer that is too small: the plan says how many rows it needs and holds nothing
    if ref["n_rows"][1] > 256:
        small = int(ref["n_rows"][1]) - 256
        Xs, ps = sf.token_pack(desc, to_dev(x, dtype), to_dev(valid, dtype), pid, Tc=small)
        torch.cuda.synchronize()
        refs = _layout_reference(valid, pattern, P, small, c)
        assert refs["n_rows"][0] == 0 and refs["n_rows"][1] == ref["n_rows"][1]
        for k in refs:
            assert np.array_equal(to_host(getattr(ps, k)), refs[k]), k
        assert not to_host(Xs).any()


def test_token_pack_pattern_out_of_range_gives_the_empty_plan():
    B, L, d, P = 6, 70, 16, 3
    rng = np.random.default_rng(3)
    valid = (rng.random((B, L)) < 0.6).astype(np.uint8)
    pattern = np.array([0, 2, 1, 3, 0, 1], np.int32)                 # 3 is not a pattern
    x = torch.from_numpy(rng.standard_normal((B, L, d)).astype(np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
    desc = sf.make_desc(B, L, d, 1, 1, 8, 8, dtype=sf.SF_BF16, P=P)
    Xp, plan = sf.token_pack(desc, to_dev(x, "bf16"), to_dev(valid, "bf16"), to_dev(pattern, "bf16"))
    torch.cuda.synchronize()
    assert to_host(plan.n_rows).tolist() == [0, -1]
    assert not to_host(plan.ext).any() and not to_host(plan.row0).any() and (to_host(plan.blk_pattern) == -1).all()
    assert (to_host(plan.src_row) == -1).all() and (to_host(plan.dst_row) == -1).all() and not to_host(Xp).any()
    assert not to_host(plan.valid_c).any() and not to_host(plan.u_active).any()
    with pytest.raises(sf.SentryFuseError):
        sf.token_pack(sf.make_desc(B, L, d, 1, 1, 8, 8, dtype=sf.SF_BF16, P=5000), to_dev(x, "bf16"), to_dev(valid, "bf16"),
                      to_dev(pattern, "bf16"))


def _packed_case(wl, samples=None, tight=True, n_sample=0):
    s = wl.spec
    bf = ORACLE_MODE[s.dtype]
    assert wl.key_valid is not None
    dm = DeviceModel(wl).build_plan()
    ref_masks = oracle_masks(wl)
    packs = compact_packs(wl, ref_masks)
    B = wl.x.shape[0]
    lens = wl.key_valid.sum(axis=1).astype(int)
    assert len(np.unique(lens)) > 1 and lens.min() < s.L        # the case really is ragged
    u_host = np.array([orc.num_active(int(t), s.c) for t in lens])
    Umax = int(u_host.max())
    pattern = wl.pattern_id.astype(np.int32)
    P = int(dm.desc.P)
    ref = _layout_reference(wl.key_valid, pattern, P, sf.token_pack_rows_max(dm.desc), s.c)
    Tc = int(ref["n_rows"][1]) if tight else sf.token_pack_rows_max(dm.desc)   # the caller knows the presence counts
    Xp, plan = sf.token_pack(dm.desc, dm.x, dm.key_valid, dm.pattern_id, Tc=Tc)
    # key sample of the sparsity score: positions of the compacted sample; those at or beyond its length count for nothing
    idx = np.random.default_rng(s.L + B).integers(0, s.L, (B, n_sample)).astype(np.int32) if n_sample else None
    idx_dev = to_dev(idx, s.dtype) if n_sample else None
    dc = desc_for(wl, U_override=Umax, n_sample=n_sample)
    Yp, sel, _ = sf.encoder_forward_packed(dc, dm.layers, Xp, plan, dm.pattern_id, final_ln=dm.final_ln, want_sel=True,
                                           sample_idx=idx_dev)
    Y = sf.token_unpack(dm.desc, Yp, plan)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(plan.len), lens) and np.array_equal(to_host(plan.u_active), u_host)
    n_rows = to_host(plan.n_rows)
    assert n_rows[1] <= Tc and n_rows[0] == n_rows[1]
    row0 = to_host(plan.row0)
    # the padded form on the same GPU: the same arithmetic row by row (its V transposition and tile walk differ)
    Lc = min(int(-(-lens.max() // 8) * 8), s.L)
    tc = sf.token_compact(dm.desc, dm.x, dm.key_valid, Lc)
    dcr = desc_for(wl, U_override=Umax, n_sample=n_sample)
    dcr.L = Lc
    Yc_pad, sel_pad, _ = sf.encoder_forward_ragged(dcr, dm.layers, tc["Xc"], dm.pattern_id, tc["valid_c"], tc["u_active"],
                                                   final_ln=dm.final_ln, want_sel=True, sample_idx=idx_dev)
    torch.cuda.synchronize()
    Yp, sel, Y, Yc_pad, sel_pad = to_host(Yp), to_host(sel), to_host(Y), to_host(Yc_pad), to_host(sel_pad)
    worst, worst_pad, picks_diff, picks_tot, sel_same = 0.0, 0.0, 0, 0, True
    for b in range(B):
        T = int(lens[b])
        keep = np.nonzero(wl.key_valid[b])[0]
        yb = Yp[row0[b]:row0[b] + T]
        assert np.isfinite(yb).all()
        # full-length output: the sample's rows at their original places, zero rows for the dropped tokens
        assert np.array_equal(Y[b, keep], yb)
        assert not Y[b, np.setdiff1d(np.arange(s.L), keep)].any()
        same = np.array_equal(sel[:, b], sel_pad[:, b])
        sel_same &= same
        if same and T:
            worst_pad = max(worst_pad, err_metric(yb, Yc_pad[b, :T]))
    for b in (range(B) if samples is None else samples):
        T, Ub = int(lens[b]), int(u_host[b])
        keep = np.nonzero(wl.key_valid[b])[0]
        xb = wl.x[b, keep][None]
        pid = wl.pattern_id[[b]]
        assert (sel[:, b, :, Ub:] == -1).all()
        fs = np.ascontiguousarray(sel[:, [b], :, :Ub])
        y_ref, _, score_f = orc.encoder_forward(xb, packs, Ub, pid, None, act=s.act, forced_sel=fs, final_ln=wl.final_ln,
                                                bf16=bf, want_score=True, sample_idx=None if idx is None else idx[[b]])
        if 0 < Ub < T:
            for l in range(s.n_layers):
                for h in range(int(wl.k_head[l])):
                    m = score_f[l, 0, h]
                    ref_sel = np.sort(np.lexsort((np.arange(T), -m.astype(np.float32)))[:Ub])
                    ok, diff = selection_report(m, sel[l, b, h, :Ub], ref_sel, None, EPS_SEL_ENC[s.dtype])
                    assert ok, (l, b, h)
                    picks_diff += len(np.setdiff1d(sel[l, b, h, :Ub], ref_sel))
                    picks_tot += Ub
        worst = max(worst, err_metric(Yp[row0[b]:row0[b] + T], y_ref[0]))
    _say(f"   packed encoder {s.name}: lens {lens.min()}..{lens.max()} (L {s.L}), rows {int(lens.sum())} in Tc {Tc} "
         f"(padded form {B * Lc}), U_b {u_host.min()}..{Umax}, err {worst:.3e}, picks differing {picks_diff}/{picks_tot}, "
         f"against the padded form {worst_pad:.3e} (same choices: {sel_same})")
    assert worst <= TOL[s.dtype], worst
    assert worst_pad <= TOL[s.dtype], worst_pad
    assert picks_diff <= max(2, int(0.03 * picks_tot)), (picks_diff, picks_tot)
    if s.dtype == "f32":
        assert picks_diff == 0
    return worst


@pytest.mark.parametrize("kw,tight", [
    (dict(dtype="f32", dropout="upto:2", B=5), True),
    (dict(dtype="f32", dropout="upto:2", B=4, nl=2, act=1, c=2), False),
    (dict(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90, 40), B=6, dropout="upto:2"), True),
    (dict(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64, 120), B=5, nl=2, dropout="upto:3", act=1), False),
    # runs of several 256-row blocks, blocks that straddle samples, more samples than one scan chunk has lanes
    (dict(dtype="bf16", d=64, dh=32, Hq=4, Hk=2, F=192, seg=(260, 140, 120, 60), B=23, nl=2, dropout="upto:2", c=1), True),
    (dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(130, 70, 60), B=40, dropout="upto:2"), True),
])
def test_encoder_packed_parity_small(kw, tight):
    _say(f"packed encoder {kw}")
    _packed_case(make_wl(W.small_spec(**kw)), tight=tight)


def test_encoder_packed_parity_with_sampled_score():
    """The sampled-key sparsity score on packed rows: the key sample is gathered from the sample's own rows."""
    _say("packed encoder, sampled score")
    _packed_case(make_wl(W.small_spec(dtype="bf16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64, 120), B=7, nl=2,
                                      dropout="upto:3", act=1)), n_sample=40)
    _packed_case(make_wl(W.small_spec(dtype="f32", dropout="upto:2", B=5)), n_sample=9)


def test_encoder_packed_parity_C3_samples():
    """The dropout workload at full size (4 modalities of 256/128/64/32 tokens, up to two dropped) in the launch
    configuration the benchmark times; the oracle on one sample of every length, every sample against the padded
    form."""
    _say("packed encoder C3")
    wl = make_wl(W.CONFIGS["C3"])
    lens = wl.key_valid.sum(axis=1)
    pick = [int(np.nonzero(lens == t)[0][-1]) for t in np.unique(lens)]
    _packed_case(wl, samples=pick[:8])


def test_packed_entry_rejects_what_it_cannot_run():
    wl = make_wl(W.small_spec(dtype="f32", dropout="upto:2", B=3))
    dm = DeviceModel(wl).build_plan()
    with pytest.raises(sf.SentryFuseError):
        sf.token_pack(dm.desc, dm.x, dm.key_valid, dm.pattern_id, Tc=300)          # not a multiple of 256
    Xp, plan = sf.token_pack(dm.desc, dm.x, dm.key_valid, dm.pattern_id)
    dc = desc_for(wl, U_override=wl.spec.L)                 # U >= L: every row active, no per-sample counts
    with pytest.raises(sf.SentryFuseError):
        sf.encoder_forward_packed(dc, dm.layers, Xp, plan, dm.pattern_id, final_ln=dm.final_ln)
    with pytest.raises(sf.SentryFuseError):
        sf.encoder_forward_packed(dm.desc, dm.layers, Xp, plan, dm.pattern_id, final_ln=dm.final_ln,
                                  ws=sf.workspace(256))                            # workspace too small


def test_pack_encode_unpack_under_hip_graph_replay():
    """Packing, the encoder over the packed rows and the unpacking recorded into one HIP graph: every replay, with
    eager work and synchronisations in between, reproduces the eager result (no step of the chain needs the host)."""
    _say("packed tokens graph replay")
    wl = make_wl(W.small_spec(dtype="bf16", d=64, dh=32, F=192, seg=(70, 50, 90, 40), B=6, dropout="upto:2"))
    s = wl.spec
    dm = DeviceModel(wl).build_plan()
    lens = wl.key_valid.sum(axis=1).astype(int)
    dc = desc_for(wl, U_override=max(orc.num_active(int(t), s.c) for t in lens))
    Tc = sf.token_pack_rows_max(dm.desc)
    plan = sf.TokenPackPlan(wl.x.shape[0], s.L, Tc, dm.x.device)
    ws = sf.workspace(sf.encoder_packed_workspace_bytes(dc, dm.layers, Tc))
    Xp = torch.empty((Tc, s.d), dtype=dm.x.dtype, device=dm.x.device)
    Yp = torch.empty_like(Xp)
    Y = torch.empty_like(dm.x)

    def chain():
        sf.token_pack(dm.desc, dm.x, dm.key_valid, dm.pattern_id, plan=plan, out=Xp)
        sf.encoder_forward_packed(dc, dm.layers, Xp, plan, dm.pattern_id, final_ln=dm.final_ln, ws=ws, out=Yp)
        return sf.token_unpack(dm.desc, Yp, plan, out=Y)

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
        chain()
    torch.cuda.synchronize()
    for rep in range(4):
        Y.fill_(float("nan"))
        ws.zero_()
        Xp.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_eager), f"replay {rep} differs from the eager result"
        Y.zero_()
        assert torch.equal(chain(), y_eager)
        torch.cuda.synchronize()
