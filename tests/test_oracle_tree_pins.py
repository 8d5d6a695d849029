"""Pins of the oracle's decode-with-draft-tree functions (CPU only).

They tie draft_step_tree / kv_append / ancestor_mask to things other than
themselves: a hand-written tree fixture, scalar brute force, the already
pinned plain draft step on truncated caches, the training forward, and
invariances that any correct masked attention has."""
import math
import os

import numpy as np
import pytest

from oracle import beagle_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _problem(M, n_true, T, H=4, G=2, d=8, D=16, seed=0):
    r = np.random.default_rng(seed)
    x = r.standard_normal((M, D))
    kc = r.standard_normal((n_true + T, G, d))
    vc = r.standard_normal((n_true + T, G, d))
    wq = r.standard_normal((D, H * d)) * 0.3
    wo = r.standard_normal((H * d, D)) * 0.3
    return x, kc, vc, wq, wo


def _read_tree_fixture():
    parents, rows = None, []
    for line in open(os.path.join(GOLD, "tree_small.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "parents":
            parents = [int(v) for v in t[1:]]
        elif t[0] == "row":
            rows.append([int(v) for v in t[2:]])
    return parents, np.array(rows, bool)


def test_ancestor_mask_matches_hand_written_tree():
    parents, want = _read_tree_fixture()
    got = orc.ancestor_mask(parents, list(range(len(parents))))
    assert got.shape == want.shape and np.array_equal(got, want)


def test_ancestor_mask_brute_force_random_trees():
    r = np.random.default_rng(3)
    for _ in range(50):
        T = int(r.integers(1, 12))
        parents = [int(r.integers(-1, t)) for t in range(T)]
        got = orc.ancestor_mask(parents, list(range(T)))
        # reachability by repeated squaring of the parent relation, written independently
        adj = np.zeros((T, T), bool)
        for t, p in enumerate(parents):
            if p >= 0:
                adj[t, p] = True
        reach = adj.copy()
        for _ in range(T):
            reach = reach | ((reach.astype(int) @ adj.astype(int)) > 0)
        assert np.array_equal(got, reach)
        assert not np.any(np.diag(got))                      # never the node itself
        assert not np.any(np.triu(got, 0))                   # only earlier nodes


def test_ancestor_mask_rejects_forward_parents():
    with pytest.raises(ValueError):
        orc.ancestor_mask([0], [0])
    with pytest.raises(ValueError):
        orc.ancestor_mask([-1, 3, 0, 0], [1])


def test_tree_step_scalar_brute_force():
    M, n_true, T, H, G, d, D = 3, 5, 4, 4, 2, 4, 6
    x, kc, vc, wq, wo = _problem(M, n_true, T, H, G, d, D, seed=1)
    tm = np.array([[1, 0, 0, 1], [0, 0, 0, 0], [1, 1, 1, 1]], bool)
    ref = orc.draft_step_tree(x, kc, vc, wq, wo, n_true=n_true, tree_mask=tm, n_q_heads=H, n_kv_heads=G)
    L = n_true + T
    y = [[0.0] * D for _ in range(M)]
    for m in range(M):
        oh = [[0.0] * d for _ in range(H)]
        for h in range(H):
            g = h // (H // G)
            q = [sum(x[m][i] * wq[i][h * d + c] for i in range(D)) for c in range(d)]
            vis = [j for j in range(L) if j < n_true or tm[m][j - n_true]]
            sc = [sum(q[c] * kc[j][g][c] for c in range(d)) / math.sqrt(d) for j in vis]
            mx = max(sc)
            e = [math.exp(v - mx) for v in sc]
            tot = sum(e)
            assert abs(ref["lse"][h][m] - (mx + math.log(tot))) < 1e-12
            for c in range(d):
                oh[h][c] = sum(e[i] / tot * vc[j][g][c] for i, j in enumerate(vis))
        flat = [oh[h][c] for h in range(H) for c in range(d)]
        for n in range(D):
            y[m][n] = sum(flat[i] * wo[i][n] for i in range(H * d))
    assert np.max(np.abs(ref["y"] - np.array(y))) < 1e-12


def test_tree_step_reduces_to_plain_step_on_truncated_caches():
    """Empty mask == plain step over the true rows; chain mask == plain step over
    the true rows plus the first m drafted rows (query m alone)."""
    M, n_true, T = 5, 9, 5
    x, kc, vc, wq, wo = _problem(M, n_true, T, seed=2)
    kw = dict(n_q_heads=4, n_kv_heads=2)
    none = orc.draft_step_tree(x, kc, vc, wq, wo, n_true=n_true, tree_mask=np.zeros((M, T), bool), **kw)
    base = orc.draft_step(x, kc[:n_true], vc[:n_true], wq, wo, **kw)
    assert np.max(np.abs(none["y"] - base["y"])) < 1e-13 and np.max(np.abs(none["lse"] - base["lse"])) < 1e-13
    chain = np.tril(np.ones((M, T), bool), -1)               # query m sees drafted rows 0 .. m-1
    got = orc.draft_step_tree(x, kc, vc, wq, wo, n_true=n_true, tree_mask=chain, **kw)
    for m in range(M):
        one = orc.draft_step(x[m:m + 1], kc[:n_true + m], vc[:n_true + m], wq, wo, **kw)
        assert np.max(np.abs(got["y"][m] - one["y"][0])) < 1e-13
        assert np.max(np.abs(got["lse"][:, m] - one["lse"][:, 0])) < 1e-13


def test_tree_step_ignores_masked_rows_bitwise_and_is_permutation_invariant():
    M, n_true, T = 4, 6, 7
    x, kc, vc, wq, wo = _problem(M, n_true, T, seed=4)
    r = np.random.default_rng(5)
    tm = r.random((M, T)) < 0.5
    kw = dict(n_true=n_true, n_q_heads=4, n_kv_heads=2)
    a = orc.draft_step_tree(x, kc, vc, wq, wo, tree_mask=tm, **kw)
    # rows of attention weights sum to one over the visible rows: uniform values => output is the mean
    kc2, vc2 = kc.copy(), vc.copy()
    hidden_everywhere = ~tm.any(axis=0)
    kc2[n_true:][hidden_everywhere] += 100.0                  # rows no query sees
    vc2[n_true:][hidden_everywhere] -= 100.0
    b = orc.draft_step_tree(x, kc2, vc2, wq, wo, tree_mask=tm, **kw)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["lse"], b["lse"])
    perm = r.permutation(T)
    kc3, vc3 = kc.copy(), vc.copy()
    kc3[n_true:], vc3[n_true:] = kc[n_true:][perm], vc[n_true:][perm]
    c = orc.draft_step_tree(x, kc3, vc3, wq, wo, tree_mask=tm[:, perm], **kw)
    assert np.max(np.abs(a["y"] - c["y"])) < 1e-12 and np.max(np.abs(a["lse"] - c["lse"])) < 1e-12


def test_kv_append_scalar_brute_force_and_untouched_rows():
    r = np.random.default_rng(6)
    cap, G, d, D, n, pos = 10, 2, 3, 5, 3, 4
    kc, vc = r.standard_normal((cap, G, d)), r.standard_normal((cap, G, d))
    xn = r.standard_normal((n, D))
    wk, wv = r.standard_normal((D, G * d)), r.standard_normal((D, G * d))
    k2, v2 = orc.kv_append(kc, vc, pos, xn, wk, wv, n_kv_heads=G)
    for i in range(cap):
        for g in range(G):
            for c in range(d):
                if pos <= i < pos + n:
                    wantk = sum(xn[i - pos][t] * wk[t][g * d + c] for t in range(D))
                    wantv = sum(xn[i - pos][t] * wv[t][g * d + c] for t in range(D))
                    assert abs(k2[i, g, c] - wantk) < 1e-12 and abs(v2[i, g, c] - wantv) < 1e-12
                else:
                    assert k2[i, g, c] == kc[i, g, c] and v2[i, g, c] == vc[i, g, c]
    with pytest.raises(ValueError):
        orc.kv_append(kc, vc, cap - 1, xn, wk, wv, n_kv_heads=G)


def test_appended_cache_reproduces_training_forward_rows():
    """Cache built by kv_append from the target states + a plain step with the
    first ws(p) rows == row p of the masked training forward (train/inference
    equivalence of section 4.1)."""
    r = np.random.default_rng(7)
    S, D, H, G, d, k, eps = 12, 8, 4, 2, 4, 3, 1
    xq, xkv = r.standard_normal((1, S, D)), r.standard_normal((1, S, D))
    wq, wk, wv = (r.standard_normal((D, n)) * 0.4 for n in (H * d, G * d, G * d))
    wo = r.standard_normal((H * d, D)) * 0.4
    mask = orc.dense_mask(S, S, k, eps)
    fw = orc.xattn_forward(xq, xkv, wq, wk, wv, wo, n_q_heads=H, n_kv_heads=G, mask=mask)
    kc, vc = np.zeros((S, G, d)), np.zeros((S, G, d))
    for start in range(0, S, 5):                              # appended in pieces
        kc, vc = orc.kv_append(kc, vc, start, xkv[0, start:start + 5], wk, wv, n_kv_heads=G)
    for p in range(S):
        n = int(mask[p].sum())
        if n == 0:
            continue
        one = orc.draft_step(xq[0, p:p + 1], kc[:n], vc[:n], wq, wo, n_q_heads=H, n_kv_heads=G)
        assert np.max(np.abs(one["y"][0] - fw["y"][0, p])) < 1e-12
