"""The allocation-free draft step (beagle_xattn_draft_step_static: scratch in the library's device image instead of
a caller-provided workspace) against beagle_xattn_draft_step on the same inputs: same kernels, so the results must
agree bit for bit -- on two calls in a row, the second with a smaller input (the shared buffer then still holds the
first call's partial sums), and in both storage types."""
import numpy as np
import pytest
import torch

from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth
import gpu_harness as gh

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(M, L, H, G, D, seed, dtype="bf16"):
    hd = 128 if dtype == "bf16" else 64
    cfg = synth.CONFIGS["c4"].with_(seq_q=M, seq_kv=L, hidden=D, n_q_heads=H, n_kv_heads=G, head_dim=hd, dtype=dtype)
    g = torch.Generator(device=DEV).manual_seed(seed)
    dt = gh.tdtype(cfg)
    R = lambda *s, std=1.0: (torch.randn(*s, device=DEV, generator=g) * std).to(dt)
    return cfg, (R(M, D), R(L, G, hd, std=1.28), R(L, G, hd, std=1.28), R(D, H * hd, std=0.02), R(H * hd, D, std=0.02))


def _both(cfg, t):
    M, D, H = cfg.seq_q, cfg.hidden, cfg.n_q_heads
    dt = gh.tdtype(cfg)
    desc = gh.desc_of(cfg)
    out = []
    for static in (False, True):
        y = torch.full((M, D), float("nan"), dtype=dt, device=DEV)
        lse = torch.full((H, M), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            bx.beagle_xattn_draft_step_static(desc, *t, y, lse)
        else:
            bx.beagle_xattn_draft_step(desc, *t, y, lse, gh.workspace(desc, bx.BEAGLE_WS_DRAFT))
        torch.cuda.synchronize()
        out.append((y, lse))
    return out


def _same(a, b):
    (y0, l0), (y1, l1) = a, b
    assert bool(torch.isfinite(y0.float()).all()) and bool(torch.isfinite(l0).all())
    assert torch.equal(y0.view(torch.int16) if y0.dtype == torch.bfloat16 else y0.view(torch.int32),
                       y1.view(torch.int16) if y1.dtype == torch.bfloat16 else y1.view(torch.int32))
    assert torch.equal(l0.view(torch.int32), l1.view(torch.int32))


def test_two_calls_in_a_row_the_second_smaller_bf16():
    big, tb = _problem(64, 4096, 32, 32, 4096, 1)          # the largest decode configuration: 26 MB of scratch
    small, ts = _problem(3, 700, 4, 2, 512, 2)
    _same(*_both(big, tb))
    _same(*_both(small, ts))
    # and straight after one another on the shared buffer, no other call in between
    db, ds = gh.desc_of(big), gh.desc_of(small)
    yb = torch.empty(64, 4096, dtype=torch.bfloat16, device=DEV); lb = torch.empty(32, 64, dtype=torch.float32, device=DEV)
    ys = torch.empty(3, 512, dtype=torch.bfloat16, device=DEV); ls = torch.empty(4, 3, dtype=torch.float32, device=DEV)
    bx.beagle_xattn_draft_step_static(db, *tb, yb, lb)
    bx.beagle_xattn_draft_step_static(ds, *ts, ys, ls)
    torch.cuda.synchronize()
    _same((yb, lb), _both(big, tb)[0])
    _same((ys, ls), _both(small, ts)[0])


def test_two_calls_in_a_row_the_second_smaller_fp32():
    big, tb = _problem(40, 300, 4, 2, 256, 3, "f32")
    small, ts = _problem(2, 50, 4, 4, 256, 4, "f32")
    _same(*_both(big, tb))
    _same(*_both(small, ts))


def test_sizes_beyond_the_static_buffer_are_refused_and_nothing_runs():
    cfg, t = _problem(64, 256, 64, 64, 8192, 5)
    desc = gh.desc_of(cfg)
    assert bx.beagle_xattn_workspace_bytes(desc, bx.BEAGLE_WS_DRAFT) > bx.BEAGLE_STATIC_SCRATCH_BYTES
    y = torch.full((64, 8192), 7.0, dtype=torch.bfloat16, device=DEV)
    lse = torch.full((64, 64), 7.0, dtype=torch.float32, device=DEV)
    st = bx.beagle_xattn_draft_step_static(desc, *t, y, lse, check=False)
    torch.cuda.synchronize()
    assert st == bx.BEAGLE_ERR_WORKSPACE and bool((y == 7.0).all()) and bool((lse == 7.0).all())
    # the ordinary entry point takes the same problem with a workspace of its own
    bx.beagle_xattn_draft_step(desc, *t, y, lse, gh.workspace(desc, bx.BEAGLE_WS_DRAFT))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y.float()).all())
    # argument errors come back as for the ordinary entry point
    assert bx.beagle_xattn_draft_step_static(gh.desc_of(cfg.with_(batch=2)), *t, y, lse, check=False) == bx.BEAGLE_ERR_SHAPE
    small, ts = _problem(2, 64, 4, 4, 512, 6)
    assert bx.beagle_xattn_draft_step_static(gh.desc_of(small), ts[0], None, *ts[2:], y, lse, check=False) == bx.BEAGLE_ERR_NULL
