#!/usr/bin/env python3
"""Writes tests/golden/fullsize_<name>.npz: sampled float64 oracle outputs for
the full-size training configs, so that the GPU parity tests at full size do
not have to run minutes of float64 CPU work on every invocation.

Calls only the oracle and the seeded input generators; nothing here touches
the HIP path.  Usage (from the repo root, about 10 minutes on 8 cores):

    python tests/golden/make_fullsize_golden.py [c2 c2_peaked c3 c5]

Stored per tensor: flat indices into the FULL tensor (int64) and the oracle's
values there (float64).  Two oracle runs per config:
  * "full"  : the whole op on ONE batch element (all heads): y, lse, q, k, v, o,
              dxq, dxkv of that element are exact; with batch 1 (c5) the weight
              gradients too.
  * "group" : the op restricted to one KV head and its query heads (weights
              sliced to that group) over ALL batch elements: o, lse of the
              group and the group's rows/columns of dwq, dwk, dwv, dwo are
              exact (they do not mix heads).  Several groups per config (the
              first, the last and one in between), stored as <tensor>@g<group>.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import beagle_oracle as orc            # noqa: E402
from paper_2505_24544_amd import synth             # noqa: E402

N_SAMPLES = 6000
OUT = os.path.dirname(os.path.abspath(__file__))

PLAN = {
    # name: (config, peaked, batch element of the full run, KV groups of the group runs)
    "c2": ("c2", False, 0, (5, 0, 31)),
    "c2_peaked": ("c2", True, 3, ()),
    "c3": ("c3", False, 1, (3, 0, 7)),
    "c5": ("c5", False, 0, ()),
}


def sample(rng, shape, n=N_SAMPLES):
    size = int(np.prod(shape))
    return np.unique(rng.integers(0, size, size=min(n, size)))


def run(name):
    cname, peaked, b_full, groups = PLAN[name]
    cfg = synth.CONFIGS[cname]
    t0 = time.time()
    inp = synth.make_inputs(cfg, peaked_queries=peaked)
    B, S, L, D = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden
    H, G, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    rep = H // G
    mask = orc.dense_mask(S, L, cfg.block_size, cfg.block_offset)
    rng = np.random.default_rng(12345)
    out = {}

    def put(tname, full_shape, idx_full, values):
        out["idx_" + tname] = idx_full.astype(np.int64)
        out["val_" + tname] = np.asarray(values, np.float64)
        out["shape_" + tname] = np.asarray(full_shape, np.int64)

    # ---- full run on one batch element
    sl = slice(b_full, b_full + 1)
    r = orc.xattn_backward(inp["dy"][sl], inp["xq"][sl], inp["xkv"][sl], inp["wq"], inp["wk"], inp["wv"], inp["wo"],
                           n_q_heads=H, n_kv_heads=G, mask=mask)
    print("  [%s] full run on batch %d: %.0f s" % (name, b_full, time.time() - t0), flush=True)
    per_b = {"y": (B, S, D), "lse": (B, H, S), "q": (B, S, H, d), "k": (B, L, G, d), "v": (B, L, G, d),
             "o": (B, S, H, d), "dxq": (B, S, D), "dxkv": (B, L, D)}
    for tname, shp in per_b.items():
        sub = r[tname]                                   # shape (1, ...)
        idx = sample(rng, sub.shape)
        # always include the last rows (longest key ranges) and the first (blind) rows
        inner = int(np.prod(sub.shape[1:]))
        idx = np.unique(np.concatenate([idx, np.arange(min(64, inner)), np.arange(inner - min(64, inner), inner)]))
        put(tname, shp, idx + b_full * inner, sub.reshape(-1)[idx])
    if B == 1:
        for tname in ("dwq", "dwk", "dwv", "dwo"):
            idx = sample(rng, r[tname].shape)
            put(tname, r[tname].shape, idx, r[tname].reshape(-1)[idx])
    del r

    # ---- group runs over all batch elements
    for gi, grp in enumerate(groups):
        sfx = "" if gi == 0 else "@g%d" % grp
        t1 = time.time()
        hs = slice(grp * rep * d, (grp + 1) * rep * d)      # query-head columns of the group
        gs = slice(grp * d, (grp + 1) * d)                  # kv-head columns
        r = orc.xattn_backward(inp["dy"], inp["xq"], inp["xkv"], inp["wq"][:, hs], inp["wk"][:, gs],
                               inp["wv"][:, gs], inp["wo"][hs, :], n_q_heads=rep, n_kv_heads=1, mask=mask)
        print("  [%s] group run (kv head %d): %.0f s" % (name, grp, time.time() - t1), flush=True)
        # o and lse of the group's heads, all batches
        o_idx = sample(rng, r["o"].shape)
        bb, pp, hh, cc = np.unravel_index(o_idx, r["o"].shape)
        put("o_group" + sfx, (B, S, H, d), np.ravel_multi_index((bb, pp, hh + grp * rep, cc), (B, S, H, d)),
            r["o"].reshape(-1)[o_idx])
        l_idx = sample(rng, r["lse"].shape)
        bb, hh, pp = np.unravel_index(l_idx, r["lse"].shape)
        put("lse_group" + sfx, (B, H, S), np.ravel_multi_index((bb, hh + grp * rep, pp), (B, H, S)),
            r["lse"].reshape(-1)[l_idx])
        # weight-gradient slices
        for tname, full_shape, col0, is_rows in (("dwq", (D, H * d), grp * rep * d, False),
                                                 ("dwk", (D, G * d), grp * d, False),
                                                 ("dwv", (D, G * d), grp * d, False),
                                                 ("dwo", (H * d, D), grp * rep * d, True)):
            g_ = r[tname]
            idx = sample(rng, g_.shape)
            i0, i1 = np.unravel_index(idx, g_.shape)
            if is_rows:
                full_idx = np.ravel_multi_index((i0 + col0, i1), full_shape)
            else:
                full_idx = np.ravel_multi_index((i0, i1 + col0), full_shape)
            put(tname + sfx, full_shape, full_idx, g_.reshape(-1)[idx])
        del r
    out["meta"] = np.array([b_full, groups[0] if groups else -1, int(peaked)], np.int64)
    path = os.path.join(OUT, "fullsize_%s.npz" % name)
    np.savez_compressed(path, **out)
    print("wrote %s (%.0f KB) in %.0f s" % (path, os.path.getsize(path) / 1e3, time.time() - t0), flush=True)


if __name__ == "__main__":
    for n in (sys.argv[1:] or list(PLAN)):
        run(n)
