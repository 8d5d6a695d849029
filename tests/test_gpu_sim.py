"""GPU parity of the late-stage simulation step (section 4.2, second half):
keys from the true states under the early-stage mask plus the predicted-state
buffer's band of the query's own window, forward and backward, against the
float64 oracle."""
import numpy as np
import pytest

from oracle import beagle_oracle as orc
from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth
from gpu_harness import run_sim, run_sim_save, run_sim_loop, run_fwd, run_bwd, max_abs, rel_fro, rel_max

pytestmark = pytest.mark.gpu
F32_TOL = 1e-5
BF16_OUT_ABS, BF16_OUT_FRO, LSE_TOL, BF16_GRAD_FRO = 2e-2, 1e-2, 1e-3, 3e-2
GRADS = ("dxq", "dxkv", "dxpred", "dwq", "dwk", "dwv", "dwo")


def _inputs(cfg, peaked=False):
    inp = synth.make_inputs(cfg, peaked_queries=peaked)
    # predicted states: the recipe of the target states with another seed (stored values of the io dtype)
    xp = synth.make_inputs(cfg.with_(seed_base=cfg.seed_base + 50), with_dy=False)["xkv"]
    return inp, xp


def _oracle(cfg, inp, xp, t):
    return orc.xattn_backward_sim(inp["dy"], inp["xq"], inp["xkv"], xp, inp["wq"], inp["wk"], inp["wv"], inp["wo"],
                                  n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, k=cfg.block_size,
                                  eps=cfg.block_offset, t=t)


@pytest.mark.parametrize("kw,t", [
    (dict(seq_q=40, seq_kv=40, block_size=4), 1), (dict(seq_q=40, seq_kv=40, block_size=4), 3),
    (dict(seq_q=40, seq_kv=40, block_size=4), 9),                          # more steps than the window holds
    (dict(batch=2, seq_q=70, seq_kv=70, n_q_heads=4, n_kv_heads=2, block_size=5, block_offset=3), 2),
    (dict(seq_q=33, seq_kv=33, block_size=8, block_offset=7), 5),
    (dict(seq_q=20, seq_kv=20, block_size=1), 3),                          # k = 1: no band at any step
    (dict(seq_q=6, seq_kv=6, block_size=8, block_offset=5), 4),            # true part blind everywhere: band only
])
def test_fp32_simulation_step(kw, t):
    cfg = synth.CONFIGS["c1"].with_(seed_base=21, **kw)
    inp, xp = _inputs(cfg)
    ref = _oracle(cfg, inp, xp, t)
    fw, gr = run_sim(cfg, inp, xp, t)
    for n in ("y", "q", "k", "v", "kp", "vp", "o"):
        assert rel_max(fw[n], ref[n]) <= F32_TOL, (n, rel_max(fw[n], ref[n]))
    fin = np.isfinite(ref["lse"])
    assert np.array_equal(np.isneginf(fw["lse"]), ~fin)
    if fin.any():
        assert max_abs(fw["lse"][fin], ref["lse"][fin]) <= F32_TOL * max(1.0, float(np.abs(ref["lse"][fin]).max()))
    for n in GRADS:
        assert rel_max(gr[n], ref[n]) <= F32_TOL, (n, rel_max(gr[n], ref[n]))
    used = orc.sim_pred_mask(cfg.seq_q, cfg.seq_kv, cfg.block_size, cfg.block_offset, t).any(axis=0)
    assert (gr["dxpred"][:, ~used] == 0).all()                               # unseen predicted rows: exactly zero


SMALL = dict(hidden=512, n_q_heads=4, n_kv_heads=4)


@pytest.mark.parametrize("name,kw,t,peaked", [
    ("c2", dict(batch=2, seq_q=300, seq_kv=300, **SMALL), 1, False),
    ("c2", dict(batch=1, seq_q=300, seq_kv=300, **SMALL), 3, True),
    ("c2", dict(batch=1, seq_q=257, seq_kv=257, block_size=5, block_offset=2, **SMALL), 2, True),
    ("c3", dict(batch=1, seq_q=330, seq_kv=330, hidden=512, n_q_heads=8, n_kv_heads=2), 7, True),
    ("c3", dict(batch=2, seq_q=260, seq_kv=260, hidden=512, n_q_heads=4, n_kv_heads=1, block_offset=5), 4, False),
])
def test_bf16_simulation_step(name, kw, t, peaked):
    cfg = synth.CONFIGS[name].with_(**kw)
    inp, xp = _inputs(cfg, peaked)
    ref = _oracle(cfg, inp, xp, t)
    fw, gr = run_sim(cfg, inp, xp, t)
    for n in ("y", "q", "k", "v", "kp", "vp", "o"):
        assert np.isfinite(fw[n]).all(), n
        assert max_abs(fw[n], ref[n]) <= BF16_OUT_ABS, (n, max_abs(fw[n], ref[n]))
        assert rel_fro(fw[n], ref[n]) <= BF16_OUT_FRO, (n, rel_fro(fw[n], ref[n]))
    fin = np.isfinite(ref["lse"])
    assert np.array_equal(np.isneginf(fw["lse"]), ~fin)
    assert max_abs(fw["lse"][fin], ref["lse"][fin]) <= (4e-3 if peaked else LSE_TOL)
    for n in GRADS:
        assert np.isfinite(gr[n]).all(), n
        assert rel_fro(gr[n], ref[n]) <= BF16_GRAD_FRO, (n, rel_fro(gr[n], ref[n]))
    used = orc.sim_pred_mask(cfg.seq_q, cfg.seq_kv, cfg.block_size, cfg.block_offset, t).any(axis=0)
    assert (gr["dxpred"][:, ~used] == 0).all()


def test_step_zero_equals_the_early_stage_entry_points_bitwise():
    cfg = synth.CONFIGS["c2"].with_(batch=1, seq_q=200, seq_kv=200, **SMALL)
    inp, xp = _inputs(cfg)
    fw, gr = run_sim(cfg, inp, xp, 0)
    dev, fw0 = run_fwd(cfg, inp)
    _, gr0 = run_bwd(cfg, inp, dev)
    for n in ("y", "lse", "o"):
        assert np.array_equal(fw[n], fw0[n], equal_nan=True), n
    for n in ("dxq", "dxkv", "dwq", "dwo"):
        assert np.array_equal(gr[n], gr0[n]), n
    assert not gr["dxpred"].any()


def test_simulation_argument_errors():
    import torch
    d = bx.make_desc(batch=1, seq_q=16, seq_kv=32, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, block_size=4,
                     io_dtype=bx.BEAGLE_F32)
    a = torch.zeros(1 << 16, device="cuda:0")
    st = bx.beagle_xattn_fwd_sim(d, a, a, a, a, a, a, a, 1, a, a, a, a, a, a, a, a, None, check=False)
    assert st == bx.BEAGLE_ERR_SHAPE                                         # seq_q != seq_kv
    d2 = bx.make_desc(batch=1, seq_q=16, seq_kv=16, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, block_size=4,
                      io_dtype=bx.BEAGLE_F32)
    assert bx.beagle_xattn_fwd_sim(d2, a, a, a, a, a, a, a, -1, a, a, a, a, a, a, a, a, None, check=False) == bx.BEAGLE_ERR_SHAPE
    assert bx.beagle_xattn_fwd_sim(d2, a, a, None, a, a, a, a, 1, a, a, a, a, a, a, a, a, None, check=False) == bx.BEAGLE_ERR_NULL


@pytest.mark.parametrize("name,kw,steps", [
    ("c1", dict(batch=2, seq_q=37, seq_kv=37, block_size=4), 6),
    ("c1", dict(batch=1, seq_q=50, seq_kv=50, block_size=5, block_offset=3), 5),
    ("c1", dict(batch=1, seq_q=9, seq_kv=9, block_size=1), 2),
    ("c2", dict(batch=2, seq_q=130, seq_kv=130, block_size=8, block_offset=5, **SMALL), 8),
])
def test_save_of_predicted_states_is_bit_exact(name, kw, steps):
    cfg = synth.CONFIGS[name].with_(seed_base=33, **kw)
    inp, xp = _inputs(cfg)
    h = inp["xkv"][:, ::-1].copy()                                           # any tensor of the buffer's shape
    for t in range(steps):
        ref = orc.sim_save_predicted(xp, h, cfg.block_size, cfg.block_offset, t)
        got = run_sim_save(cfg, h, xp, t)
        assert np.array_equal(got, ref), t
        assert (t >= cfg.block_size) == np.array_equal(got, np.asarray(xp, np.float64))


@pytest.mark.parametrize("name,kw,tol", [
    ("c1", dict(batch=2, seq_q=45, seq_kv=45, block_size=4, block_offset=1), None),
    ("c2", dict(batch=1, seq_q=200, seq_kv=200, block_size=4, **SMALL), (BF16_OUT_ABS, BF16_OUT_FRO)),
])
def test_three_simulated_steps_with_in_place_saves(name, kw, tol):
    """fwd_sim(t) -> save y as the predicted states -> fwd_sim(t + 1) ..., all on the device, against the same loop
    over the oracle; the buffer starts with large values: a step that read a row before it was saved would show."""
    cfg = synth.CONFIGS[name].with_(seed_base=44, **kw)
    inp, _ = _inputs(cfg)
    steps = 3
    init = inp["xkv"] * 64.0                                                # exact in the storage type
    buf, ref = init.astype(np.float64), []
    for t in range(steps):
        y = orc.xattn_forward_sim(inp["xq"], inp["xkv"], buf, inp["wq"], inp["wk"], inp["wv"], inp["wo"],
                                  n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, k=cfg.block_size,
                                  eps=cfg.block_offset, t=t)["y"]
        ref.append(y)
        buf = orc.sim_save_predicted(buf, y, cfg.block_size, cfg.block_offset, t)
    ys, xp = run_sim_loop(cfg, inp, init, steps)
    for t in range(steps):
        if tol is None:
            assert rel_max(ys[t], ref[t]) <= 2 * F32_TOL, (t, rel_max(ys[t], ref[t]))
        else:
            assert max_abs(ys[t], ref[t]) <= tol[0] and rel_fro(ys[t], ref[t]) <= tol[1], (t, rel_fro(ys[t], ref[t]))
    assert not np.allclose(ref[0], ref[2])                                   # the steps differ where a band exists
    assert (rel_max(xp, buf) <= 2 * F32_TOL) if tol is None else (rel_fro(xp, buf) <= tol[1])


def test_save_argument_errors():
    import torch
    a = torch.zeros(1 << 14, device="cuda:0")
    d = bx.make_desc(batch=1, seq_q=16, seq_kv=32, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, block_size=4,
                     io_dtype=bx.BEAGLE_F32)
    assert bx.beagle_xattn_sim_save(d, a, a, 0, check=False) == bx.BEAGLE_ERR_SHAPE
    d2 = bx.make_desc(batch=1, seq_q=16, seq_kv=16, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, block_size=4,
                      io_dtype=bx.BEAGLE_F32)
    assert bx.beagle_xattn_sim_save(d2, a, a, -1, check=False) == bx.BEAGLE_ERR_SHAPE
    assert bx.beagle_xattn_sim_save(d2, None, a, 0, check=False) == bx.BEAGLE_ERR_NULL


def test_rows_saved_by_later_steps_do_not_change_this_step_bitwise():
    """The rows that step t and later steps will overwrite are invisible at step t: forward results and all
    gradients are bitwise the same whatever they hold (this is what lets one buffer serve every step)."""
    cfg = synth.CONFIGS["c2"].with_(batch=1, seq_q=150, seq_kv=150, block_size=5, block_offset=2, **SMALL)
    inp, xp = _inputs(cfg)
    t = 2
    pos = (np.arange(cfg.seq_kv) - cfg.block_offset) % cfg.block_size           # position inside the window
    xp2 = xp.copy()
    xp2[:, pos >= t] = xp[:, pos >= t] * -8.0
    fw, gr = run_sim(cfg, inp, xp, t)
    fw2, gr2 = run_sim(cfg, inp, xp2, t)
    for n in ("y", "lse", "o"):
        assert np.array_equal(fw[n], fw2[n], equal_nan=True), n
    for n in GRADS:
        assert np.array_equal(gr[n], gr2[n]), n


def test_fullsize_simulation_step_on_sampled_rows():
    """The 7B-shaped training workload at step t = 3 (what bench.py's late_stage_sim object times): y and dxq of
    sampled query rows of one batch entry against the oracle evaluated on those rows over the concatenated
    [true | predicted] keys."""
    cfg = synth.CONFIGS["c2"].with_(seed_base=85, batch=2)
    inp, xp = _inputs(cfg, peaked=True)
    t, b = 3, 1
    S, L, k = cfg.seq_q, cfg.seq_kv, cfg.block_size
    d = bx.make_desc(batch=cfg.batch, seq_q=S, seq_kv=L, hidden=cfg.hidden, n_q_heads=cfg.n_q_heads,
                     n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, block_size=k, io_dtype=bx.BEAGLE_BF16,
                     flags=bx.BEAGLE_FLAG_NEED_DXKV)
    import torch
    from gpu_harness import to_dev, to_host, workspace, DEV
    B, D, H, G, hd = cfg.batch, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    dev = {n: to_dev(inp[n], cfg) for n in ("xq", "xkv", "wq", "wk", "wv", "wo", "dy")}
    dev["xp"] = to_dev(xp, cfg)
    E = lambda *s, dtype=torch.bfloat16: torch.empty(*s, dtype=dtype, device=DEV)
    y, lse, q, o = E(B, S, D), E(B, H, S, dtype=torch.float32), E(B, S, H, hd), E(B, S, H, hd)
    kk, vv, kp, vp = (E(B, L, G, hd) for _ in range(4))
    bx.beagle_xattn_fwd_sim(d, dev["xq"], dev["xkv"], dev["xp"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], t, y, lse, q,
                            kk, vv, kp, vp, o, workspace(d, bx.BEAGLE_WS_FWD))
    dxq, dxkv, dxp = E(B, S, D), E(B, L, D), E(B, L, D)
    dwq, dwk, dwv, dwo = E(D, H * hd), E(D, G * hd), E(D, G * hd), E(H * hd, D)
    bx.beagle_xattn_bwd_sim(d, dev["dy"], dev["xq"], dev["xkv"], dev["xp"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], q, kk,
                            vv, kp, vp, o, lse, t, dxq, dxkv, dxp, dwq, dwk, dwv, dwo, workspace(d, bx.BEAGLE_WS_BWD_SIM))
    torch.cuda.synchronize()
    rows = np.array([0, 1, 3, 4, 5, 6, 7, 127, 128, 129, 1023, 1025, 1026, 2046, 2047])
    mask = np.concatenate([orc.dense_mask(S, L, k, 0), orc.sim_pred_mask(S, L, k, 0, t)], axis=1)[rows]
    f64 = lambda a: np.asarray(a, np.float64)
    cat = np.concatenate([f64(inp["xkv"])[b:b + 1], f64(xp)[b:b + 1]], axis=1)
    ref = orc.xattn_backward(f64(inp["dy"])[b:b + 1, rows], f64(inp["xq"])[b:b + 1, rows], cat, inp["wq"], inp["wk"], inp["wv"],
                             inp["wo"], n_q_heads=H, n_kv_heads=G, mask=mask)
    got_y, got_dxq, got_lse = to_host(y[b, rows]), to_host(dxq[b, rows]), to_host(lse[b][:, rows])
    assert max_abs(got_y, ref["y"][0]) <= BF16_OUT_ABS and rel_fro(got_y, ref["y"][0]) <= BF16_OUT_FRO
    fin = np.isfinite(ref["lse"][0])
    assert np.array_equal(np.isneginf(got_lse), ~fin) and max_abs(got_lse[fin], ref["lse"][0][fin]) <= 1.5e-2
    assert rel_fro(got_dxq, ref["dxq"][0]) <= BF16_GRAD_FRO, rel_fro(got_dxq, ref["dxq"][0])
    # rows that hold no predicted state at this step, or that no later query of their window can see, get exactly zero
    used = orc.sim_pred_mask(S, L, k, 0, t).any(axis=0)
    assert not to_host(dxp[:, ~used]).any() and to_host(dxp[:, used]).any()
