"""GPU parity of the FP8-arithmetic pruned FFN (E4M3 codes on both operands of the two contractions) against
the CPU oracle, through the C ABI.

Bar: the plain quantiser and the compacted code buffers bit-exact; where no rounding can occur anywhere (small
integers, power-of-two scales) codes and outputs bit-exact, which pins the operand layout of the matrix
instruction; on random data the output within max |a-b| / max(1,|b|) <= 2e-2, and the codes - decided from
fp32 values that differ from the oracle's by accumulation rounding only - equal except for a small fraction of
neighbouring codes.
"""
from __future__ import annotations

import math

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as orc
from paper_2604_08971_amd import binding as sf
from gpu_utils import to_dev, to_host
from helpers import err_metric, make_wl

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _bf16(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def _cast_e4m3(a):
    """PyTorch's cast as the offline weight quantiser (inputs inside +-448)."""
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_quantize_fp8_bit_exact():
    _say("quantize_fp8")
    rng = np.random.default_rng(60)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    grid = np.array([orc.fp8_e4m3_decode(int(c)) for c in codes], np.float32)
    pos = np.sort(grid[grid > 0])
    mids = ((pos[:-1].astype(np.float64) + pos[1:]) / 2).astype(np.float32)
    edge = np.concatenate([grid, mids, -mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)),
                           np.float32([448.0, 449.0, 463.9, 464.0, 480.0, 1e9, -1e9, np.inf, -np.inf, np.nan, 0.0, -0.0,
                                       2.0 ** -10, -(2.0 ** -10), 2.0 ** -11, 1e-30, -1e-30])])
    x = np.concatenate([edge, (rng.standard_normal(100003) * 40).astype(np.float32),
                        (rng.standard_normal(50000) * 0.01).astype(np.float32)])
    for scale in (1.0, 0.0371, 3.0):
        xs = (x * np.float32(scale)).astype(np.float32) if scale == 1.0 else x
        got = to_host(sf.quantize_fp8(to_dev(xs, "f32"), scale))
        assert np.array_equal(got, orc.quantize_fp8(xs, scale)), scale
        xb = _bf16(xs)
        gotb = to_host(sf.quantize_fp8(to_dev(xb, "bf16"), scale))
        assert np.array_equal(gotb, orc.quantize_fp8(xb, scale)), scale
    # sizes around the 8-element groups, and nothing at all
    for n in (0, 1, 7, 8, 9, 2047, 2049):
        xs = x[:n].copy()
        got = to_host(sf.quantize_fp8(to_dev(xs, "f32"), 0.5))
        assert np.array_equal(got, orc.quantize_fp8(xs, 0.5))


def _case(seed, B, L, d, F, P, kf, act=0, exact=False):
    rng = np.random.default_rng(seed)
    if exact:
        # multiples of 1/4 and 1/2 with few non-zeros per row: every product, sum and quantiser input is exact
        x = _bf16(rng.integers(-2, 3, (B, L, d)) / 2.0)
        W1 = np.where(rng.random((F, d)) < 8.0 / d, rng.integers(-2, 3, (F, d)), 0) / 2.0
        W2 = np.where(rng.random((F, d)) < 8.0 / F, rng.integers(-2, 3, (F, d)), 0) / 2.0
        b1, b2 = rng.integers(-2, 3, F) / 2.0, rng.integers(-2, 3, d) / 2.0
        g = b = None
        s1 = s2 = 0.25
        sx, sh = 0.125, 0.0625
    else:
        x = _bf16(rng.standard_normal((B, L, d)) * 1.5 + 0.3)
        W1 = rng.standard_normal((F, d)) / math.sqrt(d)
        W2 = rng.standard_normal((F, d)) / math.sqrt(F)
        b1, b2 = _bf16(rng.standard_normal(F) * 0.2), _bf16(rng.standard_normal(d) * 0.1)
        g, b = _bf16(1 + 0.1 * rng.standard_normal(d)), _bf16(0.1 * rng.standard_normal(d))
        s1, s2 = float(np.float32(np.abs(W1).max() / 448)), float(np.float32(np.abs(W2).max() / 448))
        sx, sh = 4.0 / 448, 5.0 / 448          # a few values beyond 4 sigma saturate
    W1q, W2q = _cast_e4m3(W1 / np.float32(s1)), _cast_e4m3(W2 / np.float32(s2))
    keep = np.stack([np.sort(rng.choice(F, kf, replace=False)) for _ in range(P)]).astype(np.int32)
    ffn_idx = np.full((1, P, F), -1, np.int32)
    ffn_idx[0, :, :kf] = keep
    pid = rng.integers(0, P, B).astype(np.int32)
    return dict(x=x, W1q=W1q, W2q=W2q, b1=_bf16(b1), b2=_bf16(b2), g=g, b=b, s1=s1, s2=s2, sx=sx, sh=sh, keep=keep,
                ffn_idx=ffn_idx, pid=pid, B=B, L=L, d=d, F=F, P=P, kf=kf, act=act)


def _device(c, pre_ln, residual):
    desc = sf.make_desc(c["B"], c["L"], c["d"], 1, 1, 8, c["F"], 1, c["P"], sf.SF_BF16, act=c["act"])
    d8 = dict(W1=to_dev(c["W1q"], "bf16"), W2=to_dev(c["W2q"], "bf16"), b1=to_dev(c["b1"], "bf16"),
              b2=to_dev(c["b2"], "bf16"), ln2_g=to_dev(c["g"], "bf16"), ln2_b=to_dev(c["b"], "bf16"))
    masks = dict(ffn_idx=to_dev(c["ffn_idx"], "bf16"))
    cf = sf.compact_ffn_fp8(desc, 0, d8, dict(W1=c["s1"], W2=c["s2"]), masks, c["kf"], c["sx"], c["sh"])
    y, xq, hq = sf.pruned_ffn_fp8_forward(desc, cf, to_dev(c["x"], "bf16"), to_dev(c["pid"], "bf16"), pre_ln=pre_ln,
                                          add_residual=residual, want_codes=True)
    torch.cuda.synchronize()
    return cf, to_host(y), to_host(xq), to_host(hq)


def _rows_by_pattern(c, rows):
    pid_of = c["pid"][rows // c["L"]]
    return {p: rows[pid_of == p] for p in range(c["P"]) if (pid_of == p).any()}


def _all_rows(c):
    return _rows_by_pattern(c, np.arange(c["B"] * c["L"], dtype=np.int64))


def _oracle(c, p, rows, pre_ln, residual, xq_forced=None, hq_forced=None, want_z=False):
    """The oracle on the given token rows (all of pattern p).  hq_forced in the compact channel order."""
    x2 = c["x"].reshape(-1, c["d"])
    k = c["keep"][p]
    mask = np.zeros(c["F"], np.uint8)
    mask[k] = 1
    hf = None
    if hq_forced is not None:
        hf = np.zeros((rows.size, c["F"]), np.uint8)
        hf[:, k] = hq_forced
    r = orc.pruned_ffn_fp8(x2[rows], c["W1q"], c["s1"], c["b1"], c["W2q"], c["s2"], c["b2"], c["g"], c["b"], c["sx"],
                           c["sh"], ffn_mask=mask, act=c["act"], pre_ln=pre_ln, add_residual=residual, bf16=True,
                           xq_forced=xq_forced, hq_forced=hf, want_z=want_z)
    return (r[0], r[1], r[2][:, k]) + ((r[3][:, k],) if want_z else ())


def _compacted_ok(c, cf):
    Fp8 = cf.Fp8
    assert Fp8 % 128 == 0 and Fp8 - 128 < c["kf"] <= Fp8
    W1q, W2Tq, b1 = to_host(cf.W1q), to_host(cf.W2Tq), to_host(cf.b1)
    for p in range(c["P"]):
        k = c["keep"][p]
        assert np.array_equal(W1q[p, :c["kf"]], c["W1q"][k]) and not W1q[p, c["kf"]:].any()
        assert np.array_equal(W2Tq[p, :, :c["kf"]], c["W2q"][k].T) and not W2Tq[p, :, c["kf"]:].any()
        assert np.array_equal(b1[p, :c["kf"]], c["b1"][k]) and not b1[p, c["kf"]:].any()


DEC = np.array([orc.fp8_e4m3_decode(i) if (i & 0x7F) != 0x7F else 0.0 for i in range(256)])


def _neighbours(a, b):
    """codes a, b of fp32 values that differ by rounding noise: equal, or adjacent on the E4M3 grid"""
    key = lambda q: np.where(q & 0x80, -(q & 0x7F).astype(np.int32), (q & 0x7F).astype(np.int32))
    return np.abs(key(a) - key(b)) <= 1


def _act(z, act):
    if act == 0:
        return np.maximum(z, 0.0)
    return 0.5 * z * (1.0 + np.vectorize(math.erf)(z / math.sqrt(2.0)))


def _compare(c, got, pre_ln, residual, rows_of, exact):
    """A code is a floating-point decision, so the block is checked in three steps, each against the oracle:
    (1) the input codes against the oracle's own (bit-exact without LayerNorm; after LayerNorm the fp32 statistics
        differ from the fp64 ones by rounding noise, which moves a value across a grid midpoint now and then);
    (2) the hidden codes against the oracle's z computed from the DEVICE's input codes: the decoded code must lie
        within half a grid step of act(z), plus the rounding noise of an fp32 sum of K products
        (K * 2^-23 * sum |products|: the matrix instruction adds in fp32, measured 2^-17 of that sum at K = 256);
    (3) the output against the oracle run on the device's input and hidden codes: the bar of the bf16 path.
    With `exact` nothing rounds anywhere and every step is bit for bit against the oracle's free run."""
    y, xq, hq = got
    y2 = y.reshape(-1, c["d"])
    worst, flips_x, flips_h, n_x, n_h = 0.0, 0, 0, 0, 0
    for p, rows in rows_of.items():
        gx, gh = xq[rows], hq[rows][:, :c["kf"]]
        assert not hq[rows][:, c["kf"]:].any()                          # padding channels: code 0
        ry, rxq, rhq = _oracle(c, p, rows, pre_ln, residual)
        if exact:
            assert np.array_equal(gx, rxq) and np.array_equal(gh, rhq)
            assert np.array_equal(y2[rows], _bf16(ry))
            continue
        # (1)
        if not pre_ln:
            assert np.array_equal(gx, rxq)
        assert _neighbours(gx, rxq).all()
        flips_x += int((gx != rxq).sum()); n_x += gx.size
        # (2)
        _, _, rhq2, z = _oracle(c, p, rows, pre_ln, residual, xq_forced=gx, want_z=True)
        k = c["keep"][p]
        os1 = float(np.float32(np.float32(c["sx"]) * np.float32(c["s1"])))
        s_abs = (np.abs(DEC[gx]) @ np.abs(DEC[c["W1q"][k]]).T) * os1
        noise = c["d"] * 2.0 ** -23 * s_abs * 1.13                     # 1.13: largest slope of erf-GELU
        h = np.clip(_act(z, c["act"]), -448 * c["sh"], 448 * c["sh"])
        half_step = np.maximum(np.abs(h) * 2.0 ** -4, c["sh"] * 2.0 ** -10)
        dev_h = DEC[gh] * c["sh"]
        assert (np.abs(dev_h - h) <= half_step * (1 + 1e-6) + noise).all()
        flips_h += int((gh != rhq2).sum()); n_h += gh.size
        # (3)
        ry3, _, _ = _oracle(c, p, rows, pre_ln, residual, xq_forced=gx, hq_forced=gh)
        worst = max(worst, err_metric(y2[rows], ry3))
        # and against the oracle's free run the output differs only where a hidden code flipped: small on average
        assert np.sqrt(np.mean((y2[rows] - ry) ** 2)) <= 1e-2 * max(1.0, np.sqrt(np.mean(ry ** 2)))
    if not exact:
        assert flips_x <= 2e-4 * n_x + 2 and flips_h <= 2e-3 * n_h + 2, (flips_x, n_x, flips_h, n_h)
        assert worst <= 2e-2, worst
    return worst


@pytest.mark.parametrize("kw", [
    dict(B=3, L=300, d=256, F=640, P=2, kf=300),                      # ragged row tile, ragged column tile
    dict(B=2, L=520, d=384, F=900, P=3, kf=513, act=1),               # GELU, three K steps up, five down
    dict(B=1, L=192, d=256, F=256, P=1, kf=129),                      # the smallest accepted shape
    dict(B=5, L=256, d=512, F=1024, P=2, kf=1024),                    # nothing pruned, exact tiles
    dict(B=1, L=200, d=1280, F=384, P=1, kf=200),                     # wide rows: four chunks per lane in the LayerNorm
    dict(B=2, L=193, d=2176, F=256, P=2, kf=129),                     # eight chunks per lane, 17 K steps up
])
@pytest.mark.parametrize("pre_ln,residual", [(True, True), (False, False)])
def test_pruned_ffn_fp8_parity_small(kw, pre_ln, residual):
    _say(f"ffn fp8 {kw} pre_ln={pre_ln} residual={residual}")
    c = _case(61, **kw)
    cf, y, xq, hq = _device(c, pre_ln, residual)
    _compacted_ok(c, cf)
    _compare(c, (y, xq, hq), pre_ln, residual, _all_rows(c), exact=False)


@pytest.mark.parametrize("kw", [dict(B=2, L=300, d=256, F=512, P=2, kf=333), dict(B=1, L=512, d=768, F=1024, P=1, kf=900)])
def test_pruned_ffn_fp8_exact_when_nothing_rounds(kw):
    """Every code, product, sum and quantiser input is exactly representable: any difference is a wrong operand
    (a k permuted on one side only, a transposed tile, a wrong byte order in the packed conversion)."""
    _say(f"ffn fp8 exact {kw}")
    c = _case(62, exact=True, **kw)
    cf, y, xq, hq = _device(c, False, True)
    assert hq.any() and (hq > 0x40).any()                             # the case is not trivially zero
    _compare(c, (y, xq, hq), False, True, _all_rows(c), exact=True)


def test_pruned_ffn_fp8_C5_full_size_sampled():
    """The FFN of the headline workload (B 64, L 1024, d 768, 2150 of 3072 channels, 2 patterns) in the launch
    configuration the benchmark times; the oracle on 96 sampled token rows (first, last, tile borders, random)."""
    _say("ffn fp8 C5 sampled")
    c = _case(63, B=64, L=1024, d=768, F=3072, P=2, kf=2150)
    cf, y, xq, hq = _device(c, True, True)
    rng = np.random.default_rng(64)
    rows = np.unique(np.concatenate([[0, 255, 256, 1023, 1024, 65535, 65280, 65279], rng.integers(0, 65536, 88)]))
    _compare(c, (y, xq, hq), True, True, _rows_by_pattern(c, rows), exact=False)
    # padding columns of the hidden codes are zero everywhere, not only in the sampled rows
    assert not hq[:, c["kf"]:].any()


def test_pruned_ffn_fp8_rejects_what_it_cannot_run():
    c = _case(65, B=1, L=192, d=256, F=256, P=1, kf=200)
    desc = sf.make_desc(1, 192, 256, 1, 1, 8, 256, 1, 1, sf.SF_BF16)
    d8 = dict(W1=to_dev(c["W1q"], "bf16"), W2=to_dev(c["W2q"], "bf16"), b1=to_dev(c["b1"], "bf16"),
              b2=to_dev(c["b2"], "bf16"), ln2_g=to_dev(c["g"], "bf16"), ln2_b=to_dev(c["b"], "bf16"))
    masks = dict(ffn_idx=to_dev(c["ffn_idx"], "bf16"))
    cf = sf.compact_ffn_fp8(desc, 0, d8, dict(W1=c["s1"], W2=c["s2"]), masks, c["kf"], c["sx"], c["sh"])
    x = to_dev(c["x"], "bf16")
    for bad in (sf.make_desc(1, 100, 256, 1, 1, 8, 256, 1, 1, sf.SF_BF16),       # too few tokens
                sf.make_desc(1, 192, 256, 1, 1, 8, 256, 1, 1, sf.SF_F32)):       # fp32 model dtype
        with pytest.raises(sf.SentryFuseError):
            sf.pruned_ffn_fp8_forward(bad, cf, x)
    cf.struct.sh = 0.0
    with pytest.raises(sf.SentryFuseError):
        sf.pruned_ffn_fp8_forward(desc, cf, x)


# ------------------------------------------------------------- the encoder with FP8 FFNs
def _encoder_fp8_case(kw):
    from paper_2604_08971_amd import workloads as W
    from gpu_utils import DeviceModel
    from helpers import dense_packs, oracle_masks
    wl = make_wl(W.small_spec(**kw))
    s = wl.spec
    dm = DeviceModel(wl).build_plan()
    ref_masks = oracle_masks(wl)
    packs = dense_packs(wl, ref_masks)                 # dense weights + channel masks: the codes are dense too
    U = sf.num_active(dm.desc)
    B, L, d, F, nl = wl.x.shape[0], s.L, s.d, s.F, s.n_layers
    sx, sh = 4.0 / 448, 4.0 / 448
    f8, cfs = [], []
    for l in range(nl):
        lw = wl.layers[l]
        s1, s2 = float(np.float32(np.abs(lw["W1"]).max() / 448)), float(np.float32(np.abs(lw["W2"]).max() / 448))
        W1q, W2q = _cast_e4m3(lw["W1"] / np.float32(s1)), _cast_e4m3(lw["W2"] / np.float32(s2))
        f8.append(dict(W1q=W1q, W2q=W2q, s1=s1, s2=s2, sx=sx, sh=sh))
        d8 = dict(dm.dense[l], W1=to_dev(W1q, "bf16"), W2=to_dev(W2q, "bf16"))
        cfs.append(sf.compact_ffn_fp8(dm.desc, l, d8, dict(W1=s1, W2=s2), dm.masks, int(wl.k_ffn[l]), sx, sh))
    Y, sel, xq, hq = sf.encoder_forward_fp8ffn(dm.desc, dm.layers, cfs, dm.x, dm.pattern_id, dm.key_valid, dm.final_ln,
                                               want_sel=True, want_codes=True)
    torch.cuda.synchronize()
    Y, sel, xq = to_host(Y), to_host(sel), to_host(xq).reshape(nl, B, L, d)
    # the device's hidden codes in the dense channel layout of each sample's pattern
    hq_dense = np.zeros((nl, B, L, F), np.uint8)
    for l in range(nl):
        kf = int(wl.k_ffn[l])
        h = to_host(hq[l]).reshape(B, L, -1)
        assert not h[:, :, kf:].any()
        for b in range(B):
            hq_dense[l, b][:, ref_masks["ffn_idx"][l, int(wl.pattern_id[b]), :kf]] = h[b, :, :kf]
    bf = True
    # the device lists the active queries per kept head (rank order); the dense packs index heads by their number
    sel_dense = np.full((nl, B, s.Hq, U), -1, np.int32)
    for l in range(nl):
        kh = int(wl.k_head[l])
        for b in range(B):
            sel_dense[l, b, ref_masks["head_idx"][l, int(wl.pattern_id[b]), :kh]] = sel[l, b, :kh]
    common = dict(act=s.act, final_ln=wl.final_ln, bf16=bf, ffn8=f8, forced_sel=sel_dense)
    # the oracle on the device's decisions (active queries, codes): the output reference
    y_ref, _, _ = orc.encoder_forward(wl.x, packs, U, wl.pattern_id, wl.key_valid, xq_forced=xq, hq_forced=hq_dense, **common)
    e = err_metric(Y, y_ref)
    # the decisions themselves, layer by layer: the oracle's own input codes of layer l on the device's decisions of
    # the layers before it, then its own hidden codes of layer l on the device's input codes of layer l
    xq_own, hq_own = np.zeros_like(xq), np.zeros_like(hq_dense)
    for l in range(nl):
        forced = dict(xq_forced=xq, hq_forced=hq_dense, want_codes=True, **common)
        xq_own[l] = orc.encoder_forward(wl.x, packs, U, wl.pattern_id, wl.key_valid, n_forced_x=l, n_forced_h=l,
                                        **forced)[3][l]
        hq_own[l] = orc.encoder_forward(wl.x, packs, U, wl.pattern_id, wl.key_valid, n_forced_x=l + 1, n_forced_h=l,
                                        **forced)[4][l]
    vx_d, vx_o = DEC[xq] * sx, DEC[xq_own] * sx
    # the streams differ by the bf16 path's rounding noise, the codes by at most that plus one grid step
    assert (np.abs(vx_d - vx_o) <= 2.0 ** -3 * np.abs(vx_o) + 2e-2 * np.maximum(1.0, np.abs(vx_o))).all()
    vh_d, vh_o = DEC[hq_dense] * sh, DEC[hq_own] * sh
    assert (np.abs(vh_d - vh_o) <= 2.0 ** -3 * np.abs(vh_o) + 2e-3).all()
    same = float((hq_dense == hq_own).mean())
    _say(f"   encoder with fp8 ffn: err {e:.3e}; hidden codes equal to the oracle's on the device's input codes: {same:.5f}; "
         f"input codes equal to the oracle's own: {float((xq == xq_own).mean()):.4f}")
    assert same >= 0.995
    assert e <= 2e-2, e


@pytest.mark.parametrize("kw", [
    dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(100, 60, 70), extra=2, B=3, nl=2, ffn_keep=0.6,
         dropout="bernoulli:0.3"),
    dict(dtype="bf16", d=384, dh=32, Hq=12, Hk=4, F=640, seg=(128, 128), extra=0, B=2, nl=1, ffn_keep=0.8, act=1,
         dropout="none", final_ln=False),
    # long enough for the output projection to run on the active rows only: LN2 and the quantiser are then fused
    # with the pass that forms the residual stream
    dict(dtype="bf16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(260, 140, 120), extra=2, B=2, nl=2, ffn_keep=0.6,
         dropout="bernoulli:0.3"),
])
def test_encoder_with_fp8_ffn_parity(kw):
    _say(f"encoder fp8 ffn {kw}")
    _encoder_fp8_case(kw)


def test_ffn_fp8_under_hip_graph_replay():
    """The FP8 block (LayerNorm + quantiser, two GEMMs) recorded into a HIP graph: every replay, with eager work and
    synchronisations in between, reproduces the eager result bit for bit."""
    _say("ffn fp8 graph replay")
    c = _case(66, B=3, L=300, d=256, F=640, P=2, kf=300)
    desc = sf.make_desc(c["B"], c["L"], c["d"], 1, 1, 8, c["F"], 1, c["P"], sf.SF_BF16)
    d8 = dict(W1=to_dev(c["W1q"], "bf16"), W2=to_dev(c["W2q"], "bf16"), b1=to_dev(c["b1"], "bf16"),
              b2=to_dev(c["b2"], "bf16"), ln2_g=to_dev(c["g"], "bf16"), ln2_b=to_dev(c["b"], "bf16"))
    masks = dict(ffn_idx=to_dev(c["ffn_idx"], "bf16"))
    cf = sf.compact_ffn_fp8(desc, 0, d8, dict(W1=c["s1"], W2=c["s2"]), masks, c["kf"], c["sx"], c["sh"])
    X, pid = to_dev(c["x"], "bf16"), to_dev(c["pid"], "bf16")
    import ctypes
    ws = sf.workspace(sf.lib().sf_pruned_ffn_fp8_workspace_bytes(ctypes.byref(desc), c["kf"]))
    y_eager = sf.pruned_ffn_fp8_forward(desc, cf, X, pid, ws=ws).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sf.pruned_ffn_fp8_forward(desc, cf, X, pid, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        y_graph = sf.pruned_ffn_fp8_forward(desc, cf, X, pid, ws=ws)
    torch.cuda.synchronize()
    for rep in range(4):
        y_graph.fill_(float("nan"))
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {rep} differs from the eager result"
        assert torch.equal(sf.pruned_ffn_fp8_forward(desc, cf, X, pid, ws=ws), y_eager)
        torch.cuda.synchronize()
