"""GPU parity at the FULL sizes of the training configs, in the launch
configuration that bench.py times (bf16, dXkv requested), on sampled outputs.

The expected values are float64 oracle outputs at sampled positions, written
once by tests/golden/make_fullsize_golden.py (which calls only the oracle and
the input generators) into tests/golden/fullsize_*.npz."""
import os

import numpy as np
import pytest
import torch

from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth
import gpu_harness as gh

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")

OUT_ABS, OUT_FRO, LSE_TOL, GRAD_FRO = 2e-2, 1e-2, 1e-3, 3e-2
# Peaked-query variant (not one of the five configs): scores have std ~1.6, and the saved Q/K are rounded to
# bf16 (unit roundoff 2^-9), which moves a score by ~2.6e-3 rms.  A row with few visible keys inherits that
# directly in its LSE; 1.5e-2 is ~6 sigma of that.
LSE_TOL_PEAKED = 1.5e-2


def _gather(t: torch.Tensor, idx: np.ndarray) -> np.ndarray:
    i = torch.from_numpy(idx).to(t.device)
    return t.reshape(-1)[i].to(torch.float64).cpu().numpy()


@pytest.mark.parametrize("name", ["c2", "c2_peaked", "c3", "c5"])
def test_fullsize_sampled_parity(name):
    path = os.path.join(GOLD, "fullsize_%s.npz" % name)
    if not os.path.exists(path):
        pytest.skip("golden file %s not generated" % path)
    gold = np.load(path)
    cname = name.split("_")[0]
    cfg = synth.CONFIGS[cname]
    peaked = bool(gold["meta"][2])
    inp = synth.make_inputs(cfg, peaked_queries=peaked)
    dev, _ = gh.run_fwd_device(cfg, inp)
    grads = gh.run_bwd_device(cfg, inp, dev, flags=bx.BEAGLE_FLAG_NEED_DXKV)
    tensors = {**{n: dev[n] for n in ("y", "lse", "q", "k", "v", "o")}, **grads}
    tensors["o_group"], tensors["lse_group"] = dev["o"], dev["lse"]
    checked = 0
    for key in gold.files:
        if not key.startswith("idx_"):
            continue
        tname = key[4:]
        t = tensors[tname.split("@")[0]]                 # <tensor>@g<group>: the same tensor, another KV group's part
        assert tuple(gold["shape_" + tname]) == tuple(t.shape), tname
        got, ref = _gather(t, gold[key]), gold["val_" + tname]
        checked += 1
        if tname.startswith("lse"):
            fin = np.isfinite(ref)
            assert np.array_equal(np.isneginf(got), ~fin), tname
            tol = LSE_TOL_PEAKED if peaked else LSE_TOL
            assert gh.max_abs(got[fin], ref[fin]) <= tol, (tname, gh.max_abs(got[fin], ref[fin]))
        elif tname.startswith("d"):
            assert np.isfinite(got).all(), tname
            assert gh.rel_fro(got, ref) <= GRAD_FRO, (tname, gh.rel_fro(got, ref))
        else:
            assert np.isfinite(got).all(), tname
            assert gh.max_abs(got, ref) <= OUT_ABS, (tname, gh.max_abs(got, ref))
            assert gh.rel_fro(got, ref) <= OUT_FRO, (tname, gh.rel_fro(got, ref))
    assert checked >= 8


def test_fullsize_structure_properties_c5():
    """Properties that hold at any size, checked on the largest config: rows
    that see no key are exactly zero with LSE = -inf, keys that no query sees
    get exactly zero gradient, nothing is NaN, and a second run is bitwise equal."""
    cfg = synth.CONFIGS["c5"]
    inp = synth.make_inputs(cfg)
    dev, _ = gh.run_fwd_device(cfg, inp)
    g1 = gh.run_bwd_device(cfg, inp, dev, flags=bx.BEAGLE_FLAG_NEED_DXKV)
    k = cfg.block_size
    assert bool((dev["y"][:, :k] == 0).all()) and bool(torch.isneginf(dev["lse"][:, :, :k]).all())
    assert bool(torch.isfinite(dev["lse"][:, :, k:]).all())
    assert bool((g1["dxq"][:, :k] == 0).all())
    assert bool((g1["dxkv"][:, cfg.seq_kv - k:] == 0).all())        # the last window's keys are seen by nobody
    for t in list(g1.values()) + [dev["y"], dev["o"]]:
        assert bool(torch.isfinite(t.float()).all())
    snap = {n: t.clone() for n, t in g1.items()}
    y1 = dev["y"].clone()
    dev2, _ = gh.run_fwd_device(cfg, inp)
    g2 = gh.run_bwd_device(cfg, inp, dev2, flags=bx.BEAGLE_FLAG_NEED_DXKV)
    assert torch.equal(y1, dev2["y"])
    for n in snap:
        assert torch.equal(snap[n], g2[n]), n


def test_c3_key_value_weight_gradients_in_float_round_to_the_bf16_results():
    """At c3 (H 32 / G 8) dWk and dWv are computed as two halves of the contraction plus a pass that adds them (their
    tiles alone would leave half of the chip idle); that pass writes bf16 or, with BEAGLE_FLAG_WGRAD_F32, float.  Both
    come from the same float sums: the float results, rounded, are the bf16 results bit for bit; dWq (one launch
    either way) likewise.  The values themselves are checked against the oracle in test_fullsize_sampled_parity[c3]."""
    cfg = synth.CONFIGS["c3"]
    # the workspace says whether the split applies: 4 float partials of D x G d on top of the c2-like layout
    extra = 4 * cfg.hidden * cfg.n_kv_heads * cfg.head_dim * 4
    d3 = gh.desc_of(cfg, bx.BEAGLE_FLAG_NEED_DXKV)
    d_mha = gh.desc_of(cfg.with_(n_kv_heads=cfg.n_q_heads), bx.BEAGLE_FLAG_NEED_DXKV)
    base = lambda c: (2 * c.batch * c.seq_q * c.n_q_heads * c.head_dim * 2 + 2 * c.batch * c.seq_kv * c.n_kv_heads * c.head_dim * 2
                      + 2 * c.batch * c.n_q_heads * c.seq_q * 4)
    assert bx.beagle_xattn_workspace_bytes(d3, bx.BEAGLE_WS_BWD) >= base(cfg) + extra
    assert bx.beagle_xattn_workspace_bytes(d_mha, bx.BEAGLE_WS_BWD) < base(cfg.with_(n_kv_heads=cfg.n_q_heads)) + extra
    inp = synth.make_inputs(cfg)
    dev, _ = gh.run_fwd_device(cfg, inp)
    g16 = gh.run_bwd_device(cfg, inp, dev, flags=bx.BEAGLE_FLAG_NEED_DXKV)
    g32 = gh.run_bwd_device(cfg, inp, dev, flags=bx.BEAGLE_FLAG_NEED_DXKV | bx.BEAGLE_FLAG_WGRAD_F32)
    for n in ("dwq", "dwk", "dwv", "dwo"):
        assert g32[n].dtype == torch.float32 and g16[n].dtype == torch.bfloat16, n
        assert torch.equal(g32[n].to(torch.bfloat16), g16[n]), n
    for n in ("dxq", "dxkv"):
        assert torch.equal(g32[n], g16[n]), n
