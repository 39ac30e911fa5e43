"""GPU parity of the FP16 build of the library (libsentryfuse_f16.so: the same sources with IEEE binary16 as the
16-bit storage and matrix-core type, dtype SF_F16) against the CPU oracle in its binary16 mode, through the C ABI.

The cases and the bar are those of the bfloat16 build (same helpers): masks, indices and compaction bit-exact,
active sets by the margin rule; outputs within max |a-b| / max(1,|b|) <= 4e-3 (8 units of 2^-11: binary16 carries
three more significant bits than bfloat16, whose bar is 2e-2).
"""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as orc
from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W
from helpers import make_wl
from gpu_utils import DeviceModel, to_dev, to_host
from test_gpu_parity import _encoder_parity, _ffn_case, _gqa_case, _moe_case, _spread_samples

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _f16_library():
    with sf.use_half("f16"):
        yield


def _say(msg):
    print(msg, flush=True)


def test_f16_library_takes_f16_models_only():
    """Each build computes 16-bit models in its own type and says so when handed the other one."""
    d16 = sf.make_desc(1, 64, 64, 4, 2, 16, 128, dtype=sf.SF_F16)
    dbf = sf.make_desc(1, 64, 64, 4, 2, 16, 128, dtype=sf.SF_BF16)
    assert sf.lib().sf_num_active(C.byref(d16)) > 0
    assert sf.lib().sf_num_active(C.byref(dbf)) == -3
    assert b"libsentryfuse.so" in sf.lib().sf_last_error()
    with sf.use_half("bf16"):
        assert sf.lib().sf_num_active(C.byref(dbf)) > 0
        assert sf.lib().sf_num_active(C.byref(d16)) == -3
        assert b"libsentryfuse_f16.so" in sf.lib().sf_last_error()


@pytest.mark.parametrize("B,nH,nG,L,dh,Uo,mask,kw", [
    (2, 6, 2, 384, 32, -1, True, {}),                                   # C2-shaped (dh 32)
    (3, 4, 4, 480, 64, -1, True, dict(per_sample_map=True)),            # C3-shaped, per-sample head maps
    (1, 8, 4, 4096, 64, -1, False, dict(v_transposed=True)),            # C5-shaped: key splits, V key-contiguous
    (2, 4, 2, 333, 128, -1, True, dict(strided=True)),                  # dh 128, strided views of one buffer
    (2, 4, 2, 200, 64, 200, False, {}),                                 # dense pattern (U = L)
    (2, 3, 1, 203, 64, -1, True, dict(forced=True)),                    # caller-supplied active sets
    (2, 4, 2, 300, 32, 30, True, dict(n_sample=24)),                    # sampled-key score
    (2, 2, 2, 96, 64, 0, True, {}),                                     # U = 0
])
def test_f16_sparse_gqa_parity(B, nH, nG, L, dh, Uo, mask, kw):
    _say(f"f16 sgqa B={B} nH={nH} nG={nG} L={L} dh={dh} U={Uo} mask={mask} {kw}")
    _gqa_case("f16", B, nH, nG, L, dh, Uo, mask, seed=L * 7 + dh, **kw)


@pytest.mark.parametrize("act,B,L,d,F,keep", [(0, 4, 384, 256, 1024, 0.6), (1, 3, 203, 128, 520, 0.71),
                                               (0, 2, 4096, 768, 3072, 0.7)])
def test_f16_pruned_ffn_parity(act, B, L, d, F, keep):
    _say(f"f16 ffn act={act} B={B} L={L} d={d} F={F}")
    _ffn_case("f16", act, B, L, d, F, keep)


@pytest.mark.parametrize("kw", [
    dict(dtype="f16", d=64, dh=32, F=192, seg=(70, 50, 90), B=4),
    dict(dtype="f16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64), extra=3, B=3, nl=3, act=1, dropout="upto:2"),
    # long enough for the output projection on the active rows only
    dict(dtype="f16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(260, 140, 120), extra=2, B=2, nl=2, ffn_keep=0.6),
])
def test_f16_encoder_parity_small(kw):
    _say(f"f16 encoder small {kw}")
    _encoder_parity(make_wl(W.small_spec(**kw)))


@pytest.mark.parametrize("name,n_samples", [("C2", 12), ("C4", 6), ("C5", 4)])
def test_f16_encoder_parity_full_size_sampled(name, n_samples):
    """The configurations of the bfloat16 benchmark as FP16 models, at full size; the oracle takes the first and the
    last sample, both ends of every presence pattern and a seeded draw of the rest."""
    import dataclasses
    wl = make_wl(dataclasses.replace(W.CONFIGS[name], dtype="f16"))
    samples = _spread_samples(wl, n_samples)
    _say(f"f16 encoder {name} (full batch on the GPU, {len(samples)} samples through the oracle)")
    _encoder_parity(wl, samples=samples, own_choice=False)


def test_f16_encoder_on_packed_tokens():
    """Token compaction without padding in the FP16 build: the packed-row encoder against the oracle in its binary16
    mode, sample by sample at the sample's own length (the walk of tests/test_gpu_tokens_packed.py with the FP16 bar)."""
    import test_gpu_tokens_packed as TP
    TP.TOL["f16"], TP.EPS_SEL_ENC["f16"] = 4e-3, 2e-2
    _say("f16 packed tokens")
    TP._packed_case(make_wl(W.small_spec(dtype="f16", d=128, dh=64, Hq=8, Hk=2, F=300, seg=(100, 33, 64, 120), B=9, nl=2,
                                         dropout="upto:3", act=1)))


def test_f16_moe_ffn_parity():
    _say("f16 moe")
    wl = make_wl(W.small_spec(dtype="f16", d=128, dh=64, Hq=8, Hk=2, F=320, seg=(100, 133, 64), extra=3, B=5,
                                      act=1, dropout="upto:2"))
    _moe_case(wl, 8, 3)
    _moe_case(wl, 8, 3, forced=True)


@pytest.mark.parametrize("kw", [
    dict(dtype="f16", d=256, dh=64, Hq=4, Hk=2, F=512, seg=(100, 60, 70), extra=2, B=3, nl=2, head_keep=0.75,
         ffn_keep=0.6, dropout="bernoulli:0.3"),
    # long enough for the output projection on the active rows only
    dict(dtype="f16", d=256, dh=32, Hq=8, Hk=2, F=512, seg=(600, 300, 200), extra=0, B=2, nl=2, head_keep=0.5, c=5,
         ffn_keep=0.6, dropout="bernoulli:0.3"),
])
def test_f16_encoder_with_fp8_projections_and_ffn(kw):
    """FP8 arithmetic (projections and FFN) on top of an FP16 model: the decision-by-decision walk of the bfloat16
    build against the oracle in its binary16 mode."""
    from test_gpu_fp8_proj import _case
    _say(f"f16 encoder fp8 {kw}")
    _case(kw, True)


def test_f16_weight_storage_and_fp8_paths():
    """An FP16 model stores binary16 weights as they are (sf_compact_heads_channels_f16 is the plain gather, bit for
    bit); E4M3-stored weights, the stand-alone FP8 FFN block and the plain quantiser on 16-bit input are built for
    bfloat16 models and are refused here."""
    wl = make_wl(W.small_spec(dtype="f16", d=64, dh=32, F=192, seg=(70, 50, 90), B=3, nl=1))
    dm = DeviceModel(wl).build_plan()
    got = sf.compact_heads_channels_f16(dm.desc, 0, dm.dense[0], dm.masks, int(wl.k_head[0]), int(wl.k_ffn[0]))
    torch.cuda.synchronize()
    for name in ("Wqkv", "WoT", "W1", "W2T"):
        assert torch.equal(getattr(got, name).view(torch.int16), getattr(dm.layers[0], name).view(torch.int16)), name
    x8 = torch.zeros(64, dtype=torch.float16, device="cuda")
    codes = torch.empty(64, dtype=torch.uint8, device="cuda")
    f8 = sf.SfFfnFp8()
    f8.k_ffn, f8.s1, f8.s2, f8.sx, f8.sh = 200, 1.0, 1.0, 1.0, 1.0
    f8.W1q = f8.W2Tq = 256
    d8 = sf.make_desc(1, 256, 256, 8, 2, 32, 512, dtype=sf.SF_F16)
    args = (C.c_void_p(256), None, 1, 1, C.c_void_p(512), None, None, None, 0, None)
    assert sf.lib().sf_pruned_ffn_fp8_forward(C.byref(d8), C.byref(f8), *args) == -3
    assert b"bfloat16" in sf.lib().sf_last_error()
    assert sf.lib().sf_quantize_fp8(sf._ptr(x8), sf.SF_BF16, 64, 1.0, sf._ptr(codes), None) == -3
