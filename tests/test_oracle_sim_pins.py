"""Pins of the oracle's late-stage simulation functions (CPU only): hand-written
masks, closed-form counts, reduction to the early stage and to the decode-time
draft step over a concatenated cache, scalar brute force, finite differences."""
import math
import os

import numpy as np
import pytest

from oracle import beagle_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _fixtures():
    cases, cur = [], None
    for line in open(os.path.join(GOLD, "sim_mask_small.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "case":
            cur = dict(S=int(t[2]), k=int(t[4]), eps=int(t[6]), t=int(t[8]), rows=[])
            cases.append(cur)
        elif t[0] == "row":
            cur["rows"].append([int(v) for v in t[2:]])
    return cases


@pytest.mark.parametrize("case", _fixtures(), ids=lambda c: "k%d_eps%d_t%d" % (c["k"], c["eps"], c["t"]))
def test_pred_mask_matches_hand_written(case):
    want = np.array(case["rows"], bool)
    S = case["S"]
    assert np.array_equal(orc.sim_pred_mask_loops(S, S, case["k"], case["eps"], case["t"]), want)
    assert np.array_equal(orc.sim_pred_mask(S, S, case["k"], case["eps"], case["t"]), want)


def test_pred_mask_closed_form_equals_loops_and_counts():
    for S, L in ((1, 1), (7, 7), (16, 16), (13, 9), (9, 13)):
        for k in (1, 2, 3, 4, 5, 8):
            for eps in range(k):
                for t in range(0, k + 2):
                    a = orc.sim_pred_mask_loops(S, L, k, eps, t)
                    b = orc.sim_pred_mask(S, L, k, eps, t)
                    assert np.array_equal(a, b), (S, L, k, eps, t)
                    true = orc.dense_mask(S, L, k, eps)
                    assert not (a & true).any()                       # a key position is never visible twice
                    assert not np.triu(a, 0).any()                    # strictly before the query
                    if t == 0 or k == 1:
                        assert not a.any()
    # whole windows: each contributes sum_{i<k} min(i, t) visible predicted keys
    for S, k in ((16, 4), (24, 8), (30, 5)):
        for t in range(k + 1):
            want = (S // k) * sum(min(i, t) for i in range(k))
            assert int(orc.sim_pred_mask(S, S, k, 0, t).sum()) == want
    # t >= k-1: true + predicted keys together are exactly the strictly causal set j < p
    for k, eps in ((4, 0), (4, 3), (5, 2)):
        S = 17
        both = orc.dense_mask(S, S, k, eps) | orc.sim_pred_mask(S, S, k, eps, k - 1)
        assert np.array_equal(both, np.tri(S, S, -1, dtype=bool))


def _problem(B=1, S=10, D=6, H=4, G=2, d=3, seed=0):
    r = np.random.default_rng(seed)
    xq, xkv, xp = (r.standard_normal((B, S, D)) for _ in range(3))
    wq = r.standard_normal((D, H * d)) * 0.5
    wk, wv = r.standard_normal((D, G * d)) * 0.5, r.standard_normal((D, G * d)) * 0.5
    wo = r.standard_normal((H * d, D)) * 0.5
    dy = r.standard_normal((B, S, D))
    return xq, xkv, xp, wq, wk, wv, wo, dy


def test_step_zero_is_the_early_stage():
    xq, xkv, xp, wq, wk, wv, wo, dy = _problem(B=2, seed=1)
    kw = dict(n_q_heads=4, n_kv_heads=2)
    a = orc.xattn_backward_sim(dy, xq, xkv, xp, wq, wk, wv, wo, k=3, eps=1, t=0, **kw)
    b = orc.xattn_backward(dy, xq, xkv, wq, wk, wv, wo, mask=orc.dense_mask(10, 10, 3, 1), **kw)
    for n in ("y", "lse", "dxq", "dxkv", "dwq", "dwk", "dwv", "dwo"):
        fin = np.isfinite(b[n])
        assert np.array_equal(np.isfinite(a[n]), fin), n
        assert np.max(np.abs(a[n][fin] - b[n][fin])) < 1e-12, n      # same terms, longer (zero-padded) sums
    assert not a["dxpred"].any()


def test_forward_scalar_brute_force():
    B, S, D, H, G, d, k, eps, t = 1, 7, 4, 2, 1, 3, 3, 1, 2
    xq, xkv, xp, wq, wk, wv, wo, _ = _problem(B, S, D, H, G, d, seed=2)
    ref = orc.xattn_forward_sim(xq, xkv, xp, wq, wk, wv, wo, n_q_heads=H, n_kv_heads=G, k=k, eps=eps, t=t)
    for p in range(S):
        w0 = eps + k * math.floor((p - eps) / k)
        keys = [("t", j) for j in range(S) if j < max(w0, 0)]
        keys += [("p", j) for j in range(S) if max(w0, 0) <= j < min(p, w0 + t)]
        flat = []
        for h in range(H):
            q = [sum(xq[0][p][i] * wq[i][h * d + c] for i in range(D)) for c in range(d)]
            rows = []
            for src, j in keys:
                x = xkv[0][j] if src == "t" else xp[0][j]
                kk = [sum(x[i] * wk[i][c] for i in range(D)) for c in range(d)]    # G == 1
                vv = [sum(x[i] * wv[i][c] for i in range(D)) for c in range(d)]
                rows.append((sum(q[c] * kk[c] for c in range(d)) / math.sqrt(d), vv))
            if not rows:
                flat += [0.0] * d
                assert ref["lse"][0, h, p] == -np.inf
                continue
            mx = max(s for s, _ in rows)
            tot = sum(math.exp(s - mx) for s, _ in rows)
            assert abs(ref["lse"][0, h, p] - (mx + math.log(tot))) < 1e-12
            flat += [sum(math.exp(s - mx) / tot * vv[c] for s, vv in rows) for c in range(d)]
        y = [sum(flat[i] * wo[i][n] for i in range(H * d)) for n in range(D)]
        assert np.max(np.abs(ref["y"][0, p] - np.array(y))) < 1e-12


def test_full_simulation_row_equals_draft_step_over_concatenated_cache():
    """At t = k-1, row p is exactly what inference computes for that position: a
    plain draft step whose cache holds the true rows before the window followed
    by the drafted (predicted) rows of the window up to p (section 4.1 / 4.2:
    the simulation reproduces inference)."""
    B, S, D, H, G, d, k, eps = 1, 11, 6, 4, 2, 3, 4, 1
    xq, xkv, xp, wq, wk, wv, wo, _ = _problem(B, S, D, H, G, d, seed=3)
    kw = dict(n_q_heads=H, n_kv_heads=G)
    ref = orc.xattn_forward_sim(xq, xkv, xp, wq, wk, wv, wo, k=k, eps=eps, t=k - 1, **kw)
    for p in range(1, S):
        w0 = max(eps + k * math.floor((p - eps) / k), 0)
        states = np.concatenate([xkv[0, :w0], xp[0, w0:p]], axis=0)
        kc, vc = orc.kv_project(states, wk, wv, n_kv_heads=G)
        one = orc.draft_step(xq[0, p:p + 1], kc, vc, wq, wo, **kw)
        assert np.max(np.abs(one["y"][0] - ref["y"][0, p])) < 1e-12
        assert np.max(np.abs(one["lse"][:, 0] - ref["lse"][0, :, p])) < 1e-12


def test_hidden_predicted_rows_do_not_matter_bitwise():
    B, S, k, eps, t = 2, 12, 4, 2, 2
    xq, xkv, xp, wq, wk, wv, wo, dy = _problem(B, S, seed=4)
    kw = dict(n_q_heads=4, n_kv_heads=2, k=k, eps=eps, t=t)
    a = orc.xattn_backward_sim(dy, xq, xkv, xp, wq, wk, wv, wo, **kw)
    used = orc.sim_pred_mask(S, S, k, eps, t).any(axis=0)
    xp2 = xp.copy()
    xp2[:, ~used] += 50.0
    b = orc.xattn_backward_sim(dy, xq, xkv, xp2, wq, wk, wv, wo, **kw)
    for n in ("y", "lse", "dxq", "dxkv", "dwq", "dwk", "dwv", "dwo"):
        assert np.array_equal(a[n], b[n]), n
    assert not a["dxpred"][:, ~used].any() and a["dxpred"][:, used].any()


def test_gradients_by_finite_differences():
    B, S, D, H, G, d, k, eps, t = 1, 6, 4, 2, 1, 2, 3, 1, 2
    xq, xkv, xp, wq, wk, wv, wo, dy = _problem(B, S, D, H, G, d, seed=5)
    kw = dict(n_q_heads=H, n_kv_heads=G, k=k, eps=eps, t=t)
    g = orc.xattn_backward_sim(dy, xq, xkv, xp, wq, wk, wv, wo, **kw)

    def loss(**repl):
        a = dict(xq=xq, xkv=xkv, xpred=xp, wq=wq, wk=wk, wv=wv, wo=wo)
        a.update(repl)
        return float((orc.xattn_forward_sim(a["xq"], a["xkv"], a["xpred"], a["wq"], a["wk"], a["wv"], a["wo"], **kw)["y"] * dy).sum())

    h = 1e-6
    for name, arr, grad in (("xpred", xp, g["dxpred"]), ("xkv", xkv, g["dxkv"]), ("xq", xq, g["dxq"]),
                            ("wk", wk, g["dwk"]), ("wv", wv, g["dwv"]), ("wq", wq, g["dwq"]), ("wo", wo, g["dwo"])):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            up, dn = arr.copy(), arr.copy()
            up[i] += h
            dn[i] -= h
            num[i] = (loss(**{name: up}) - loss(**{name: dn})) / (2 * h)
        scale = max(1.0, float(np.abs(num).max()))
        assert np.max(np.abs(num - grad)) / scale < 1e-6, name


# ---------------------------------------------------------------- in-place update between steps
@pytest.mark.parametrize("L,k,eps,t,rows", [
    # written by hand from the prose: after step t the rows at position t of every window are saved
    (10, 4, 0, 0, [0, 4, 8]), (10, 4, 0, 1, [1, 5, 9]), (10, 4, 0, 3, [3, 7]), (10, 4, 0, 4, []),
    (10, 4, 2, 0, [2, 6]), (10, 4, 2, 1, [3, 7]), (10, 4, 2, 2, [0, 4, 8]), (10, 4, 2, 3, [1, 5, 9]),
    (5, 1, 0, 0, [0, 1, 2, 3, 4]), (5, 1, 0, 1, []), (3, 8, 5, 3, [0]), (3, 8, 5, 0, []),
])
def test_save_predicted_rows_hand_written(L, k, eps, t, rows):
    rng = np.random.default_rng(5)
    buf, h = rng.normal(size=(2, L, 3)), rng.normal(size=(2, L, 3))
    out = orc.sim_save_predicted(buf, h, k, eps, t)
    sel = np.zeros(L, bool)
    sel[rows] = True
    assert np.array_equal(out[:, sel], h[:, sel]) and np.array_equal(out[:, ~sel], buf[:, ~sel])
    assert np.array_equal(buf, np.asarray(buf))            # the input is not modified


@pytest.mark.parametrize("k,eps", [(4, 0), (5, 3), (8, 7), (1, 0)])
def test_saved_rows_are_exactly_what_the_next_steps_may_see(k, eps):
    """Start from a buffer of NaN; after the saves of steps 0 .. t-1 every predicted key that the mask of
    step t shows is a saved one, and no row saved later is visible yet."""
    L = 37
    h = np.ones((1, L, 1))
    buf = np.full((1, L, 1), np.nan)
    for t in range(0, k + 2):
        vis = orc.sim_pred_mask_loops(L, L, k, eps, t).any(axis=0)
        assert not np.isnan(buf[0, vis, 0]).any(), (t, np.flatnonzero(vis))
        later = np.ones((1, L, 1))
        for u in range(t, k + 2):
            later = orc.sim_save_predicted(later, np.full((1, L, 1), np.nan), k, eps, u)
        assert not (np.isnan(later[0, :, 0]) & vis).any()
        buf = orc.sim_save_predicted(buf, h, k, eps, t)
    assert not np.isnan(buf).any()                            # after k steps the buffer is full


def test_simulation_loop_never_reads_the_initial_buffer():
    """Three steps with h := y as the stand-in for the block's output: the result of every step is bitwise
    independent of what the buffer held before the first step."""
    rng = np.random.default_rng(9)
    B, S, D, H, G, k, eps = 1, 14, 8, 2, 1, 4, 1
    xq, xkv = rng.normal(size=(B, S, D)), rng.normal(size=(B, S, D))
    wq, wo = rng.normal(size=(D, D)) * 0.3, rng.normal(size=(D, D)) * 0.3
    wk, wv = rng.normal(size=(D, D // 2)) * 0.3, rng.normal(size=(D, D // 2)) * 0.3
    outs = []
    for init in (np.zeros((B, S, D)), rng.normal(size=(B, S, D)) * 100):
        buf, ys = init, []
        for t in range(3):
            y = orc.xattn_forward_sim(xq, xkv, buf, wq, wk, wv, wo, n_q_heads=H, n_kv_heads=G, k=k, eps=eps, t=t)["y"]
            ys.append(y)
            buf = orc.sim_save_predicted(buf, y, k, eps, t)
        outs.append(ys)
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    assert not np.array_equal(outs[0][0], outs[0][1])         # and the steps do differ
