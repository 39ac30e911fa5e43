"""The entry point that allocates nothing (sf_sparse_gqa_forward_static) against sf_sparse_gqa_forward: same
kernels, the scratch memory comes from the library's built-in device buffer.  Two calls in a row, the second on a
smaller problem (the buffer keeps the first call's contents), plus the size limit."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W
from gpu_utils import to_dev

pytestmark = pytest.mark.gpu


def _inputs(B, nH, nG, L, dh, seed, masked):
    rng = np.random.default_rng(seed)
    Q, K, V = (to_dev(W.to_bf16_values(rng.standard_normal(s).astype(np.float32)), "bf16")
               for s in ((B, nH, L, dh), (B, nG, L, dh), (B, nG, L, dh)))
    per = nH // nG
    hg = torch.tensor([[h // per for h in range(nH)]], dtype=torch.int32, device="cuda")
    kv = None
    if masked:
        m = (rng.random((B, L)) < 0.7).astype(np.uint8)
        m[:, 0] = 1
        kv = torch.from_numpy(m).cuda()
    return Q, K, V, hg, kv


def _both(B, nH, nG, L, dh, seed, masked, dtype=sf.SF_BF16, U_override=-1):
    Q, K, V, hg, kv = _inputs(B, nH, nG, L, dh, seed, masked)
    if dtype == sf.SF_F32:
        Q, K, V = Q.float(), K.float(), V.float()
    desc = sf.make_desc(B, L, 64, nH, nG, dh, 64, dtype=dtype, U_override=U_override)
    U = sf.num_active(desc)
    assert sf.sparse_gqa_workspace_bytes(desc, nH, nG) <= sf.sparse_gqa_static_capacity()
    O_ref, sel_ref, score_ref = sf.sparse_gqa_forward(desc, Q, K, V, hg, key_valid=kv, want_sel=True, want_score=True)
    O = torch.full_like(O_ref, float("nan"))
    sel = torch.full((B, nH, max(U, 1)), -7, dtype=torch.int32, device="cuda")
    score = torch.full((B, nH, L), float("nan"), dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_allocated()
    sf.sparse_gqa_forward_static(desc, Q, K, V, hg, O, key_valid=kv, sel=sel, score=score)
    assert torch.cuda.memory_allocated() == before          # nothing came from torch's allocator either
    torch.cuda.synchronize()
    # same kernels, same order, deterministic: bit-identical outputs
    assert torch.equal(O, O_ref), (B, nH, nG, L, dh)
    assert torch.equal(sel[:, :, :U], sel_ref)
    if 0 < U < L:
        assert torch.equal(score, score_ref)


def test_static_scratch_matches_workspace_entry_point_on_two_calls_in_a_row():
    # first a larger problem with key splits (their partial sums live in the scratch buffer) and a key mask,
    # then a smaller one, then fp32, then the larger one again
    _both(2, 6, 2, 1024, 64, seed=1, masked=True)
    _both(1, 4, 2, 200, 32, seed=2, masked=False)
    _both(2, 4, 2, 48, 16, seed=3, masked=True, dtype=sf.SF_F32)
    _both(3, 8, 4, 384, 64, seed=4, masked=False, U_override=384)      # dense pattern
    _both(2, 6, 2, 1024, 64, seed=5, masked=True)


def test_static_scratch_refuses_problems_beyond_its_size():
    B, nH, nG, L, dh = 16, 8, 4, 4096, 64
    desc = sf.make_desc(B, L, 64, nH, nG, dh, 64, dtype=sf.SF_BF16)
    assert sf.sparse_gqa_workspace_bytes(desc, nH, nG) > sf.sparse_gqa_static_capacity()
    Q = torch.zeros((B, nH, L, dh), dtype=torch.bfloat16, device="cuda")
    K = torch.zeros((B, nG, L, dh), dtype=torch.bfloat16, device="cuda")
    O = torch.zeros((B, L, nH * dh), dtype=torch.bfloat16, device="cuda")
    hg = torch.zeros((1, nH), dtype=torch.int32, device="cuda")
    with pytest.raises(sf.SentryFuseError, match="built-in buffer"):
        sf.sparse_gqa_forward_static(desc, Q, K, K, hg, O)
