"""Oracle-side plumbing (TEST INFRASTRUCTURE, like everything under oracle/): builds the
oracle's layer packs and key masks from a synthetic workload.

No arithmetic of the method lives here, only slicing and bookkeeping around
oracle.cpu_oracle.  Imported by tests/, the smoke check and the benchmark's
CPU-baseline leg only.
"""
from __future__ import annotations

import numpy as np

from oracle import cpu_oracle as orc


def key_valid_of(wl):
    """The oracle's own key mask of a workload ([B, L] uint8, Sec. 4.2 / 4.4) from its presence masks and token ->
    modality map; None when every modality is present everywhere (no mask: the same result, see the pins)."""
    if wl.presence.all():
        return None
    return orc.key_valid(wl.presence, wl.tok_modality)


def oracle_masks(wl):
    s = wl.spec
    return orc.gate_scores_to_masks(wl.g_head, wl.g_ffn, wl.k_head, wl.k_ffn, s.Hk)


def dense_packs(wl, masks):
    """packs[l][p]: full weights + 0/1 masks (the plain definition of pruning)."""
    s = wl.spec
    per = s.Hq // s.Hk
    hg = np.arange(s.Hq, dtype=np.int32) // per
    return [[orc.LayerPack(wl.layers[l], s.Hq, s.Hk, s.dh, hg,
                           masks["head_mask"][l, p], masks["ffn_mask"][l, p])
             for p in range(wl.P)] for l in range(s.n_layers)]


def compact_weights(wl, masks, l, p):
    """Row-sliced weights of layer l / pattern p, done with numpy fancy indexing."""
    s = wl.spec
    w = wl.layers[l]
    kh, kf = int(wl.k_head[l]), int(wl.k_ffn[l])
    hi = masks["head_idx"][l, p, :kh]
    fi = masks["ffn_idx"][l, p, :kf]
    ng = int(masks["n_groups"][l, p])
    gi = masks["group_idx"][l, p, :ng]
    dh = s.dh
    hrows = (hi[:, None] * dh + np.arange(dh)[None, :]).reshape(-1)
    grows = (gi[:, None] * dh + np.arange(dh)[None, :]).reshape(-1)
    c = {
        "Wq": w["Wq"][hrows], "bq": w["bq"][hrows],
        "Wk": w["Wk"][grows], "bk": w["bk"][grows],
        "Wv": w["Wv"][grows], "bv": w["bv"][grows],
        "Wo": w["Wo"][hrows], "bo": w["bo"],
        "W1": w["W1"][fi], "b1": w["b1"][fi], "W2": w["W2"][fi], "b2": w["b2"],
        "ln1_g": w["ln1_g"], "ln1_b": w["ln1_b"], "ln2_g": w["ln2_g"], "ln2_b": w["ln2_b"],
    }
    return c, kh, ng, masks["head_group"][l, p, :kh]


def compact_packs(wl, masks):
    s = wl.spec
    packs = []
    for l in range(s.n_layers):
        row = []
        for p in range(wl.P):
            c, kh, ng, hg = compact_weights(wl, masks, l, p)
            row.append(orc.LayerPack(c, kh, ng, s.dh, hg))
        packs.append(row)
    return packs


def err_metric(a, b):
    """max |a-b| / max(1,|b|): the error measure of the parity bar."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b) / np.maximum(1.0, np.abs(b)))) if a.size else 0.0
