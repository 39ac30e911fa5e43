"""A synthetic workload resident on the GPU, driven through the C-ABI binding: uploads
the arrays, derives the allowed keys from the presence masks, runs plan
construction (masks + compaction) and the encoder.  Every step of the method
runs inside the library; this module only moves arrays and keeps handles.
Used by the tests, the smoke check and the benchmark.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from paper_2604_08971_amd import binding as sf
from paper_2604_08971_amd import workloads as W


SF_DTYPE = {"f32": sf.SF_F32, "bf16": sf.SF_BF16, "f16": sf.SF_F16}
# the oracle's storage-rounding mode of each model dtype
ORACLE_MODE = {"f32": 0, "bf16": 1, "f16": 2}


def to_dev(a: Optional[np.ndarray], dtype: str, device="cuda") -> Optional[torch.Tensor]:
    """fp32 host array (bf16-valued when dtype == 'bf16') -> device tensor of the path's dtype."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32 and dtype == "bf16":
        t = t.to(torch.bfloat16)          # exact: the values are bf16 numbers already
    if t.dtype == torch.float32 and dtype == "f16":
        t = t.to(torch.float16)           # exact as well
    return t.to(device).contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    t = t.detach()
    if t.dtype in (torch.bfloat16, torch.float16):
        t = t.to(torch.float32)
    return t.cpu().numpy()


def desc_for(wl: W.Workload, B: Optional[int] = None, U_override: int = -1, c: Optional[int] = None,
             n_sample: int = 0):
    s = wl.spec
    return sf.make_desc(B=wl.x.shape[0] if B is None else B, L=s.L, d_model=s.d, Hq=s.Hq, Hk=s.Hk, dh=s.dh,
                        d_ff=s.F, n_layers=s.n_layers, P=wl.P,
                        dtype=SF_DTYPE[s.dtype], act=s.act,
                        c_factor=s.c if c is None else c, U_override=U_override,
                        final_ln=wl.final_ln is not None, n_sample=n_sample)


class DeviceModel:
    """A workload resident on the GPU: dense weights, plan (masks, compact layers), inputs."""

    def __init__(self, wl: W.Workload, U_override: int = -1, device="cuda", sample_idx: Optional[np.ndarray] = None):
        s = wl.spec
        self.wl, self.device = wl, device
        self.sample_idx = None if sample_idx is None else torch.from_numpy(
            np.ascontiguousarray(sample_idx, dtype=np.int32)).to(device)
        self.desc = desc_for(wl, U_override=U_override, n_sample=0 if sample_idx is None else sample_idx.shape[1])
        dt = s.dtype
        self.x = to_dev(wl.x, dt, device)
        self.pattern_id = to_dev(wl.pattern_id, dt, device)
        # Sec. 4.2: the allowed keys follow from the presence masks; a batch in which every modality is present
        # runs without a key mask (the same result, pinned on the oracle side)
        self.presence = to_dev(wl.presence, dt, device)
        self.tok_modality = to_dev(wl.tok_modality, dt, device)
        self.key_valid = None if bool(wl.presence.all()) else sf.presence_to_key_valid(self.presence, self.tok_modality)
        self.g_head = to_dev(wl.g_head, "f32", device)
        self.g_ffn = to_dev(wl.g_ffn, "f32", device)
        self.dense = [{k: to_dev(v, dt, device) for k, v in lw.items()} for lw in wl.layers]
        self.final_ln = None if wl.final_ln is None else {k: to_dev(v, dt, device) for k, v in wl.final_ln.items()}
        self.masks: Dict[str, torch.Tensor] = {}
        self.layers: List[sf.CompactLayer] = []
        self.ws: Optional[torch.Tensor] = None

    def build_plan(self):
        """a1 + a2: gate scores -> masks -> compacted weights, all on the GPU."""
        wl = self.wl
        first = not self.layers
        self.masks = sf.gate_scores_to_masks(self.desc, self.g_head, self.g_ffn, wl.k_head, wl.k_ffn,
                                             out=None if first else self.masks)
        self.layers = [sf.compact_heads_channels(self.desc, l, self.dense[l], self.masks,
                                                 int(wl.k_head[l]), int(wl.k_ffn[l]),
                                                 out=None if first else self.layers[l])
                       for l in range(wl.spec.n_layers)]
        return self

    def forward(self, forced_sel=None, want_sel=False, want_score=False, out=None):
        if self.ws is None:
            self.ws = sf.workspace(sf.encoder_workspace_bytes(self.desc, self.layers), self.device)
        return sf.encoder_forward(self.desc, self.layers, self.x, self.pattern_id, self.key_valid,
                                  self.final_ln, forced_sel=forced_sel, want_sel=want_sel,
                                  want_score=want_score, out=out, ws=self.ws, sample_idx=self.sample_idx)


def key_valid_host(dm: "DeviceModel") -> Optional[np.ndarray]:
    """The device's key mask on the host ([B, L] uint8), None when the batch runs without one."""
    return None if dm.key_valid is None else to_host(dm.key_valid)
