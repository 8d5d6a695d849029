"""Pins for the float64 oracle: every check compares it with something that is
not the oracle itself (hand-written fixtures from the paper's prose, closed
forms, brute-force scalar loops, a library attention routine, autograd, finite
differences, invariants).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import beagle_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng


def _rand_problem(seed, B=2, S=12, D=10, H=4, G=2, d=3, L=None):
    r = RNG(seed)
    L = S if L is None else L
    return dict(
        xq=r.standard_normal((B, S, D)), xkv=r.standard_normal((B, L, D)),
        wq=r.standard_normal((D, H * d)) * 0.4, wk=r.standard_normal((D, G * d)) * 0.4,
        wv=r.standard_normal((D, G * d)) * 0.4, wo=r.standard_normal((H * d, D)) * 0.4,
        dy=r.standard_normal((B, S, D)))


def _ws(p, k, eps):
    """Start of the window that holds query p (integer closed form)."""
    return max(0, eps + k * ((p - eps) // k))


# ------------------------------------------------------------------ mask
@pytest.mark.parametrize("name,k,eps", [("mask_k3_eps1_s8.txt", 3, 1), ("mask_k1_s5.txt", 1, 0)])
def test_mask_matches_handwritten_fixture(name, k, eps):
    want = np.loadtxt(os.path.join(GOLD, name), dtype=int).astype(bool)
    S = want.shape[0]
    assert np.array_equal(orc.dense_mask_loops(S, S, k, eps), want)
    assert np.array_equal(orc.dense_mask(S, S, k, eps), want)


def test_mask_k1_is_strict_causal():
    for S in (1, 2, 7, 33):
        m = orc.dense_mask(S, S, 1, 0)
        p, j = np.mgrid[0:S, 0:S]
        assert np.array_equal(m, j < p)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
def test_mask_vectorised_equals_loops_and_row_limit(k):
    for eps in range(k):
        for S, L in ((1, 1), (5, 5), (16, 16), (19, 19), (11, 17), (17, 11)):
            a = orc.dense_mask_loops(S, L, k, eps)
            b = orc.dense_mask(S, L, k, eps)
            assert np.array_equal(a, b)
            # each row is a prefix of length min(ws(p), L)
            for p in range(S):
                n = min(_ws(p, k, eps), L)
                assert a[p, :n].all() and not a[p, n:].any()
            # rows of one window are identical
            for p in range(1, S):
                if _ws(p, k, eps) == _ws(p - 1, k, eps):
                    assert np.array_equal(a[p], a[p - 1])


@pytest.mark.parametrize("S,k,count", [(128, 4, 7936), (2048, 4, 2093056),
                                       (4096, 8, 8372224), (8192, 8, 33521664)])
def test_mask_visible_pair_count_closed_form(S, k, count):
    assert count == S * (S - k) // 2
    assert orc.visible_pairs(orc.dense_mask(S, S, k, 0)) == count


def test_mask_rejects_bad_window():
    with pytest.raises(ValueError):
        orc.dense_mask(4, 4, 0, 0)
    with pytest.raises(ValueError):
        orc.dense_mask(4, 4, 3, 3)


# ------------------------------------------------------------------ forward
def _brute_forward(t, H, G, mask):
    """Scalar loops with math.exp: the definition, one number at a time."""
    xq, xkv, wq, wk, wv, wo = (t[n] for n in ("xq", "xkv", "wq", "wk", "wv", "wo"))
    B, S, D = xq.shape
    L = xkv.shape[1]
    d = wq.shape[1] // H
    rep = H // G
    y = np.zeros((B, S, D))
    lse = np.full((B, H, S), -np.inf)
    for b in range(B):
        for p in range(S):
            orow = [0.0] * (H * d)
            for h in range(H):
                g = h // rep
                q = [sum(xq[b, p, i] * wq[i, h * d + c] for i in range(D)) for c in range(d)]
                sc, vs = [], []
                for j in range(L):
                    if not mask[p, j]:
                        continue
                    kj = [sum(xkv[b, j, i] * wk[i, g * d + c] for i in range(D)) for c in range(d)]
                    vj = [sum(xkv[b, j, i] * wv[i, g * d + c] for i in range(D)) for c in range(d)]
                    sc.append(sum(a * b_ for a, b_ in zip(q, kj)) / math.sqrt(d))
                    vs.append(vj)
                if not sc:
                    continue
                z = sum(math.exp(s) for s in sc)
                lse[b, h, p] = math.log(z)
                for s, vj in zip(sc, vs):
                    w = math.exp(s) / z
                    for c in range(d):
                        orow[h * d + c] += w * vj[c]
            for i in range(D):
                y[b, p, i] = sum(orow[c] * wo[c, i] for c in range(H * d))
    return y, lse


@pytest.mark.parametrize("k,eps,H,G", [(1, 0, 2, 2), (2, 1, 2, 1), (3, 0, 2, 2), (4, 3, 4, 2)])
def test_forward_matches_scalar_brute_force(k, eps, H, G):
    t = _rand_problem(3 + k, B=1, S=8, D=5, H=H, G=G, d=4)
    mask = orc.dense_mask_loops(8, 8, k, eps)
    out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                            n_q_heads=H, n_kv_heads=G, mask=mask)
    y, lse = _brute_forward(t, H, G, mask)
    np.testing.assert_allclose(out["y"], y, rtol=0, atol=1e-13)
    fin = np.isfinite(lse)
    assert np.array_equal(fin, np.isfinite(out["lse"]))
    np.testing.assert_allclose(out["lse"][fin], lse[fin], rtol=0, atol=1e-13)


def test_rows_sum_to_one_and_masked_weights_are_zero():
    H, G = 4, 2
    t = _rand_problem(11, S=21, H=H, G=G)
    for k, eps in ((1, 0), (4, 0), (5, 2), (8, 7)):
        mask = orc.dense_mask(21, 21, k, eps)
        out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                                n_q_heads=H, n_kv_heads=G, mask=mask, keep_probs=True)
        P = out["p"]
        assert (P[:, :, ~mask] == 0.0).all()
        rows = mask.any(axis=1)
        np.testing.assert_allclose(P[:, :, rows].sum(-1), 1.0, rtol=0, atol=1e-15 * 40)
        # empty rows: zero output, -inf LSE, nothing NaN
        assert (P[:, :, ~rows] == 0).all()
        assert (out["o"][:, ~rows] == 0).all() and (out["y"][:, ~rows] == 0).all()
        assert np.isneginf(out["lse"][:, :, ~rows]).all()
        assert np.isfinite(out["lse"][:, :, rows]).all() and np.isfinite(out["y"]).all()


def test_prefix_reduction_to_library_attention():
    """Row p equals UNMASKED attention of Q_p over the first ws(p) keys,
    computed by torch's scaled_dot_product_attention in float64."""
    H, G, d, S, k, eps = 4, 4, 8, 24, 5, 2
    t = _rand_problem(5, B=1, S=S, D=16, H=H, G=G, d=d)
    mask = orc.dense_mask(S, S, k, eps)
    out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                            n_q_heads=H, n_kv_heads=G, mask=mask)
    q = torch.from_numpy(t["xq"][0] @ t["wq"]).reshape(S, H, d).transpose(0, 1)
    kk = torch.from_numpy(t["xkv"][0] @ t["wk"]).reshape(S, G, d).transpose(0, 1)
    vv = torch.from_numpy(t["xkv"][0] @ t["wv"]).reshape(S, G, d).transpose(0, 1)
    for p in range(S):
        n = _ws(p, k, eps)
        if n == 0:
            continue
        ref = torch.nn.functional.scaled_dot_product_attention(
            q[:, p:p + 1], kk[:, :n], vv[:, :n])            # [H,1,d]
        np.testing.assert_allclose(out["o"][0, p], ref[:, 0].numpy(), rtol=0, atol=1e-13)
        yref = ref[:, 0].reshape(-1).numpy() @ t["wo"]
        np.testing.assert_allclose(out["y"][0, p], yref, rtol=0, atol=1e-13)


def test_uniform_attention_closed_form():
    """Zero queries: every visible key gets weight 1/ws(p); LSE = ln ws(p)."""
    H, G, S, k, eps = 2, 1, 17, 4, 1
    t = _rand_problem(8, B=1, S=S, H=H, G=G)
    t["xq"][:] = 0
    mask = orc.dense_mask(S, S, k, eps)
    out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                            n_q_heads=H, n_kv_heads=G, mask=mask)
    v = (t["xkv"][0] @ t["wv"]).reshape(S, G, -1)
    for p in range(S):
        n = _ws(p, k, eps)
        if n == 0:
            continue
        for h in range(H):
            np.testing.assert_allclose(out["o"][0, p, h], v[:n, 0].mean(0), atol=1e-14)
            assert abs(out["lse"][0, h, p] - math.log(n)) < 1e-14


def test_softmax_shift_invariance_and_scale_argument():
    r = RNG(2)
    s = r.standard_normal((6, 9)) * 3
    mask = orc.dense_mask(6, 9, 2, 1)
    P0, l0 = orc.masked_softmax(s, mask)
    P1, l1 = orc.masked_softmax(s + 7.25, mask)
    rows = mask.any(1)
    np.testing.assert_allclose(P0, P1, atol=1e-15)
    np.testing.assert_allclose(l1[rows], l0[rows] + 7.25, atol=1e-13)
    # large scores do not overflow
    P2, l2 = orc.masked_softmax(s * 1e4, mask)
    assert np.isfinite(P2).all() and np.isfinite(l2[rows]).all()
    # default scale is 1/sqrt(d_h): doubling d by zero-padding heads' weights is
    # NOT the same; passing the scale explicitly is.
    t = _rand_problem(4, B=1, S=6, H=2, G=2, d=4)
    m = orc.dense_mask(6, 6, 1, 0)
    kw = dict(n_q_heads=2, n_kv_heads=2, mask=m)
    a = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], **kw)
    b = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], scale=0.5, **kw)
    np.testing.assert_allclose(a["y"], b["y"], atol=1e-15)       # 1/sqrt(4) == 0.5


def test_future_keys_do_not_leak():
    H, G, S, k, eps = 2, 2, 16, 4, 2
    t = _rand_problem(13, B=1, S=S, H=H, G=G)
    mask = orc.dense_mask(S, S, k, eps)
    kw = dict(n_q_heads=H, n_kv_heads=G, mask=mask)
    base = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], **kw)
    for j in (0, 5, 9, 15):
        x2 = t["xkv"].copy()
        x2[0, j] += 3.0
        out = orc.xattn_forward(t["xq"], x2, t["wq"], t["wk"], t["wv"], t["wo"], **kw)
        for p in range(S):
            same = np.array_equal(out["y"][0, p], base["y"][0, p])
            assert same == (_ws(p, k, eps) <= j), (p, j)


def test_key_permutation_invariance():
    H, G, S = 2, 1, 10
    t = _rand_problem(17, B=1, S=S, H=H, G=G)
    mask = orc.dense_mask(S, S, 5, 0)
    perm = np.r_[np.array([3, 1, 4, 0, 2]), np.arange(5, S)]   # shuffle inside keys 0..4
    kw = dict(n_q_heads=H, n_kv_heads=G)
    a = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], mask=mask, **kw)
    b = orc.xattn_forward(t["xq"], t["xkv"][:, perm], t["wq"], t["wk"], t["wv"], t["wo"],
                          mask=mask[:, perm], **kw)
    np.testing.assert_allclose(a["y"], b["y"], atol=1e-14)


def test_gqa_equals_mha_with_repeated_kv_heads():
    H, G, d = 6, 2, 3
    t = _rand_problem(21, H=H, G=G, d=d)
    mask = orc.dense_mask(12, 12, 3, 1)
    rep = H // G
    D = t["wk"].shape[0]
    wk_r = np.repeat(t["wk"].reshape(D, G, d), rep, axis=1).reshape(D, H * d)
    wv_r = np.repeat(t["wv"].reshape(D, G, d), rep, axis=1).reshape(D, H * d)
    a = orc.xattn_backward(t["dy"], t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                           n_q_heads=H, n_kv_heads=G, mask=mask)
    b = orc.xattn_backward(t["dy"], t["xq"], t["xkv"], t["wq"], wk_r, wv_r, t["wo"],
                           n_q_heads=H, n_kv_heads=H, mask=mask)
    for n in ("y", "lse", "dxq", "dxkv", "dwq", "dwo"):
        np.testing.assert_allclose(a[n], b[n], atol=1e-12)
    for n in ("dwk", "dwv"):   # GQA weight grads are the sum over the repeated copies
        np.testing.assert_allclose(a[n], b[n].reshape(D, G, rep, d).sum(2).reshape(D, G * d), atol=1e-12)


# ------------------------------------------------------------------ backward
GRADS = ("dxq", "dxkv", "dwq", "dwk", "dwv", "dwo")
WRT = dict(dxq="xq", dxkv="xkv", dwq="wq", dwk="wk", dwv="wv", dwo="wo")


def _loss(t, H, G, mask):
    out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                            n_q_heads=H, n_kv_heads=G, mask=mask)
    return float((out["y"] * t["dy"]).sum())


@pytest.mark.parametrize("k,eps,H,G", [(1, 0, 2, 2), (3, 1, 4, 2), (4, 0, 2, 1)])
def test_gradients_match_central_finite_differences(k, eps, H, G):
    S = 9
    t = _rand_problem(31 + k, B=2, S=S, D=6, H=H, G=G, d=3)
    mask = orc.dense_mask(S, S, k, eps)
    g = orc.xattn_backward(t["dy"], t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                           n_q_heads=H, n_kv_heads=G, mask=mask)
    step = 1e-6
    r = RNG(0)
    for gname in GRADS:
        x = t[WRT[gname]]
        idxs = [tuple(r.integers(0, n) for n in x.shape) for _ in range(25)]
        for idx in idxs:
            old = x[idx]
            x[idx] = old + step
            fp = _loss(t, H, G, mask)
            x[idx] = old - step
            fm = _loss(t, H, G, mask)
            x[idx] = old
            fd = (fp - fm) / (2 * step)
            assert abs(fd - g[gname][idx]) <= 1e-6 * max(1.0, abs(fd)), (gname, idx, fd, g[gname][idx])


def test_gradients_match_autograd_float64():
    H, G, d, S, k, eps = 4, 2, 5, 14, 4, 3
    t = _rand_problem(41, B=2, S=S, D=12, H=H, G=G, d=d)
    mask = orc.dense_mask(S, S, k, eps)
    g = orc.xattn_backward(t["dy"], t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                           n_q_heads=H, n_kv_heads=G, mask=mask)
    tt = {n: torch.tensor(t[n], dtype=torch.float64, requires_grad=True)
          for n in ("xq", "xkv", "wq", "wk", "wv", "wo")}
    B = 2
    q = (tt["xq"] @ tt["wq"]).reshape(B, S, H, d).permute(0, 2, 1, 3)
    kk = (tt["xkv"] @ tt["wk"]).reshape(B, S, G, d).permute(0, 2, 1, 3).repeat_interleave(H // G, 1)
    vv = (tt["xkv"] @ tt["wv"]).reshape(B, S, G, d).permute(0, 2, 1, 3).repeat_interleave(H // G, 1)
    s = q @ kk.transpose(-1, -2) / math.sqrt(d)
    m = torch.from_numpy(mask)
    rows = m.any(1)
    s = s.masked_fill(~m, float("-inf"))
    # rows without a visible key are left out of the softmax (they are zero rows)
    p = torch.zeros_like(s)
    p[:, :, rows] = torch.softmax(s[:, :, rows], dim=-1)
    y = (p @ vv).permute(0, 2, 1, 3).reshape(B, S, H * d) @ tt["wo"]
    (y * torch.from_numpy(t["dy"])).sum().backward()
    np.testing.assert_allclose(g["y"], y.detach().numpy(), atol=1e-13)
    for gname in GRADS:
        np.testing.assert_allclose(g[gname], tt[WRT[gname]].grad.numpy(), rtol=0, atol=1e-11)


def test_gradient_invariants():
    H, G, S, k, eps = 4, 2, 15, 4, 1
    t = _rand_problem(51, B=1, S=S, H=H, G=G)
    mask = orc.dense_mask(S, S, k, eps)
    g = orc.xattn_backward(t["dy"], t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                           n_q_heads=H, n_kv_heads=G, mask=mask)
    # keys that no query can see get exactly zero gradient
    last = _ws(S - 1, k, eps)
    assert last < S
    assert (g["dk"][0, last:] == 0).all() and (g["dv"][0, last:] == 0).all()
    assert (g["dxkv"][0, last:] == 0).all()
    # queries that see nothing get exactly zero gradient
    blind = ~mask.any(1)
    assert blind.any() and (g["dq"][0, blind] == 0).all() and (g["dxq"][0, blind] == 0).all()
    # delta_p = sum_j P_pj dP_pj  (the softmax Jacobian's row term)
    out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                            n_q_heads=H, n_kv_heads=G, mask=mask, keep_probs=True)
    for h in range(H):
        dP = g["do"][0, :, h] @ out["v"][0, :, h // (H // G)].T
        np.testing.assert_allclose(g["delta"][0, h], (out["p"][0, h] * dP).sum(-1), atol=1e-12)


# ------------------------------------------------------------------ decode
def test_draft_step_reproduces_training_rows():
    """Train/inference equivalence: query p of the masked forward equals a
    draft step against a cache holding exactly the keys visible to p."""
    H, G, d, S, k, eps = 4, 2, 4, 18, 5, 3
    t = _rand_problem(61, B=1, S=S, D=8, H=H, G=G, d=d)
    mask = orc.dense_mask(S, S, k, eps)
    out = orc.xattn_forward(t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"],
                            n_q_heads=H, n_kv_heads=G, mask=mask)
    for p in range(S):
        n = _ws(p, k, eps)
        if n == 0:
            continue
        st = orc.draft_step(t["xq"][0, p:p + 1], out["k"][0, :n], out["v"][0, :n],
                            t["wq"], t["wo"], n_q_heads=H, n_kv_heads=G)
        np.testing.assert_allclose(st["y"][0], out["y"][0, p], atol=1e-13)
        np.testing.assert_allclose(st["lse"][:, 0], out["lse"][0, :, p], atol=1e-13)


def test_draft_step_single_query_closed_form():
    r = RNG(71)
    H, G, d, L, D = 2, 1, 3, 7, 5
    x = r.standard_normal((1, D))
    kc, vc = r.standard_normal((L, G, d)), r.standard_normal((L, G, d))
    wq, wo = r.standard_normal((D, H * d)), r.standard_normal((H * d, D))
    st = orc.draft_step(x, kc, vc, wq, wo, n_q_heads=H, n_kv_heads=G)
    o = []
    for h in range(H):
        q = x[0] @ wq[:, h * d:(h + 1) * d]
        w = np.array([math.exp(float(q @ kc[j, 0]) / math.sqrt(d)) for j in range(L)])
        assert abs(st["lse"][h, 0] - math.log(w.sum())) < 1e-13
        o.append((w[:, None] * vc[:, 0]).sum(0) / w.sum())
    np.testing.assert_allclose(st["y"][0], np.concatenate(o) @ wo, atol=1e-13)


def test_draft_queries_are_independent_of_each_other():
    r = RNG(72)
    H, G, d, L, D, M = 4, 2, 4, 9, 6, 5
    x = r.standard_normal((M, D))
    kc, vc = r.standard_normal((L, G, d)), r.standard_normal((L, G, d))
    wq, wo = r.standard_normal((D, H * d)), r.standard_normal((H * d, D))
    full = orc.draft_step(x, kc, vc, wq, wo, n_q_heads=H, n_kv_heads=G)
    for m in range(M):
        one = orc.draft_step(x[m:m + 1], kc, vc, wq, wo, n_q_heads=H, n_kv_heads=G)
        np.testing.assert_allclose(one["y"][0], full["y"][m], atol=1e-14)
