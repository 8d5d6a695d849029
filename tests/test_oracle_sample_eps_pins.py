"""Pins of the per-entry window offset (CPU only; section 4.2's random offset, one per sequence)."""
import numpy as np
import pytest

from oracle import beagle_oracle as orc


def _case(B=3, S=13, D=8, H=2, G=1, seed=0):
    rng = np.random.default_rng(seed)
    d = D // H
    return dict(xq=rng.normal(size=(B, S, D)), xkv=rng.normal(size=(B, S, D)), wq=rng.normal(size=(D, H * d)) * 0.4,
                wk=rng.normal(size=(D, G * d)) * 0.4, wv=rng.normal(size=(D, G * d)) * 0.4,
                wo=rng.normal(size=(H * d, D)) * 0.4), dict(n_q_heads=H, n_kv_heads=G), rng.normal(size=(B, S, D))


def test_equal_offsets_reduce_to_the_shared_mask():
    c, kw, dy = _case()
    for eps in (0, 2):
        a = orc.xattn_backward_sample_eps(dy, **c, **kw, k=4, eps_list=[eps] * 3)
        b = orc.xattn_backward(dy, **c, **kw, mask=orc.dense_mask(13, 13, 4, eps))
        for n in ("y", "lse", "o", "dxq", "dxkv"):
            assert np.array_equal(a[n], b[n]), n
        for n in ("dwq", "dwk", "dwv", "dwo"):
            assert np.allclose(a[n], b[n], atol=1e-13), n


def test_each_entry_hides_its_own_window_hand_written():
    """k = 4, offsets (0, 1, 3): first visible key count per query written out by hand from the prose
    (entry with offset 1: windows [-3,1), [1,5), [5,9) ...; offset 3: [-1,3), [3,7), ...)."""
    c, kw, _ = _case()
    want = {0: [0, 0, 0, 0, 4, 4, 4, 4, 8, 8, 8, 8, 12],
            1: [0, 1, 1, 1, 1, 5, 5, 5, 5, 9, 9, 9, 9],
            3: [0, 0, 0, 3, 3, 3, 3, 7, 7, 7, 7, 11, 11]}
    eps_list = [0, 1, 3]
    base = orc.xattn_forward_sample_eps(**c, **kw, k=4, eps_list=eps_list)["y"]
    for b, eps in enumerate(eps_list):
        for j in range(13):
            x2 = c["xkv"].copy()
            x2[b, j] += 1.0
            y2 = orc.xattn_forward_sample_eps(**dict(c, xkv=x2), **kw, k=4, eps_list=eps_list)["y"]
            changed = np.abs(y2 - base).max(axis=-1) > 0            # [B, S]
            assert not changed[[i for i in range(3) if i != b]].any()
            assert np.array_equal(changed[b], np.array(want[eps]) > j), (eps, j)


def test_gradients_by_finite_differences_and_linearity_over_the_batch():
    c, kw, dy = _case(seed=3)
    eps_list = [2, 0, 3]
    g = orc.xattn_backward_sample_eps(dy, **c, **kw, k=4, eps_list=eps_list)
    loss = lambda cc: float((orc.xattn_forward_sample_eps(**cc, **kw, k=4, eps_list=eps_list)["y"] * dy).sum())
    rng = np.random.default_rng(4)
    for n, gn in (("xq", "dxq"), ("xkv", "dxkv"), ("wq", "dwq"), ("wk", "dwk"), ("wv", "dwv"), ("wo", "dwo")):
        d = rng.normal(size=c[n].shape)
        fd = (loss(dict(c, **{n: c[n] + 1e-6 * d})) - loss(dict(c, **{n: c[n] - 1e-6 * d}))) / 2e-6
        assert abs(fd - (g[gn] * d).sum()) <= 1e-6 * max(1.0, abs(fd)), n
    with pytest.raises(ValueError):
        orc.xattn_forward_sample_eps(**c, **kw, k=4, eps_list=[0, 1])
