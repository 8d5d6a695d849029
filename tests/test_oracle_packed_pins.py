"""Pins of the oracle's packed variable-length batches (CPU only)."""
import numpy as np
import pytest

from oracle import beagle_oracle as orc


def _w(D=8, H=2, G=1, seed=0):
    rng = np.random.default_rng(seed)
    d = D // H
    return dict(wq=rng.normal(size=(D, H * d)) * 0.4, wk=rng.normal(size=(D, G * d)) * 0.4,
                wv=rng.normal(size=(D, G * d)) * 0.4, wo=rng.normal(size=(H * d, D)) * 0.4), dict(n_q_heads=H, n_kv_heads=G)


def test_equal_lengths_are_the_batched_call():
    w, kw = _w()
    rng = np.random.default_rng(1)
    B, S, D = 3, 9, 8
    xq, xkv, dy = rng.normal(size=(B, S, D)), rng.normal(size=(B, S, D)), rng.normal(size=(B, S, D))
    cu = [0, 9, 18, 27]
    a = orc.xattn_backward_packed(dy.reshape(-1, D), xq.reshape(-1, D), xkv.reshape(-1, D), **w, cu_q=cu, cu_kv=cu, **kw, k=4)
    b = orc.xattn_backward(dy, xq, xkv, **w, **kw, mask=orc.dense_mask(S, S, 4, 0))
    for n in ("y", "dxq", "dxkv", "o"):
        assert np.array_equal(a[n], b[n].reshape(a[n].shape)), n
    assert np.array_equal(a["lse"], b["lse"].transpose(1, 0, 2).reshape(2, -1))
    for n in ("dwq", "dwk", "dwv", "dwo"):
        assert np.allclose(a[n], b[n], atol=1e-13), n


def test_sequences_do_not_see_each_other_and_masks_restart():
    """Lengths (5, 7), k = 2: perturbing key row r of sequence s changes exactly the queries of s whose window
    starts after the key's index inside s (hand-written), nothing else."""
    w, kw = _w()
    rng = np.random.default_rng(2)
    cu = [0, 5, 12]
    xq, xkv = rng.normal(size=(12, 8)), rng.normal(size=(12, 8))
    base = orc.xattn_forward_packed(xq, xkv, **w, cu_q=cu, cu_kv=cu, **kw, k=2)
    assert base["y"].shape == (12, 8) and base["lse"].shape == (2, 12)
    ws_local = {5: [0, 0, 2, 2, 4], 7: [0, 0, 2, 2, 4, 4, 6]}               # visible-key counts per local query
    for s_, (lo, n) in enumerate(((0, 5), (5, 7))):
        for j in range(n):
            x2 = xkv.copy()
            x2[lo + j] += 1.0
            y2 = orc.xattn_forward_packed(xq, x2, **w, cu_q=cu, cu_kv=cu, **kw, k=2)["y"]
            changed = np.abs(y2 - base["y"]).max(-1) > 0
            want = np.zeros(12, bool)
            want[lo:lo + n] = np.array(ws_local[n]) > j
            assert np.array_equal(changed, want), (s_, j)
    # blind queries: the first window of EVERY sequence
    assert np.array_equal(np.isneginf(base["lse"][0]), np.array([1, 1, 0, 0, 0, 1, 1, 0, 0, 0, 0, 0], bool))


def test_different_query_and_key_lengths_offsets_rope_and_gradients():
    w, kw = _w(seed=3)
    rng = np.random.default_rng(4)
    cu_q, cu_kv = [0, 4, 10], [0, 6, 9]
    xq, xkv, dy = rng.normal(size=(10, 8)), rng.normal(size=(9, 8)), rng.normal(size=(10, 8))
    args = dict(cu_q=cu_q, cu_kv=cu_kv, **kw, k=3, eps_list=[1, 2], rope=dict(base=50.0))
    g = orc.xattn_backward_packed(dy, xq, xkv, **w, **args)
    # sequence 1 alone, as a batch of one
    one = orc.xattn_backward(dy[None, 4:], xq[None, 4:], xkv[None, 6:], **w, **kw, mask=orc.dense_mask(6, 3, 3, 2), rope=dict(base=50.0))
    assert np.array_equal(g["y"][4:], one["y"][0]) and np.array_equal(g["dxkv"][6:], one["dxkv"][0])
    loss = lambda **o: float((orc.xattn_forward_packed(**{**dict(xq=xq, xkv=xkv, **w), **o}, **args)["y"] * dy).sum())
    for n, gn, ref in (("xq", "dxq", xq), ("xkv", "dxkv", xkv), ("wk", "dwk", w["wk"]), ("wo", "dwo", w["wo"])):
        d = rng.normal(size=ref.shape)
        fd = (loss(**{n: ref + 1e-6 * d}) - loss(**{n: ref - 1e-6 * d})) / 2e-6
        assert abs(fd - (g[gn] * d).sum()) <= 1e-6 * max(1.0, abs(fd)), n
    with pytest.raises(ValueError):
        orc.xattn_forward_packed(xq, xkv, **w, cu_q=[0, 4, 9], cu_kv=cu_kv, **kw, k=3)
    with pytest.raises(ValueError):
        orc.xattn_forward_packed(xq, xkv, **w, cu_q=[0, 4, 4, 10], cu_kv=[0, 6, 6, 9], **kw, k=3)     # empty sequence
