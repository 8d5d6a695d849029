"""Pins of the oracle's rotary position embedding (CPU only): an independent complex-number construction, the
relative-position property, orthogonality, special cases, torch autograd through an independently built torch
attention with rotated q/k, the decode path against the training path."""
import numpy as np
import pytest
import torch

from oracle import beagle_oracle as orc


def test_rotation_is_multiplication_by_a_unit_complex_number():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(2, 7, 3, 8))
    pos = np.array([0, 1, 2, 5, 9, 100, 4095])
    base = 10000.0
    z = (x[..., :4] + 1j * x[..., 4:]) * np.exp(1j * pos[:, None, None] * base ** (-np.arange(4) / 4.0)[None, None, :])
    got = orc.rope_rotate(x, pos, base)
    assert np.allclose(got[..., :4], z.real, atol=1e-12) and np.allclose(got[..., 4:], z.imag, atol=1e-12)
    # hand values: d = 2, one pair, angle = position (base^0 = 1): position pi/2 turns (1, 0) into (0, 1)
    assert np.allclose(orc.rope_rotate(np.array([[[1.0, 0.0]]]), [np.pi / 2]), [[[0.0, 1.0]]], atol=1e-15)
    # second pair of d = 4 turns at base^(-1/2) of the first one's rate
    r = orc.rope_rotate(np.array([[[1.0, 1.0, 0.0, 0.0]]]), [3.0], base=100.0)
    assert np.allclose(r, [[[np.cos(3.0), np.cos(0.3), np.sin(3.0), np.sin(0.3)]]], atol=1e-15)


def test_position_zero_is_identity_norms_are_kept_inverse_undoes():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 2, 16))
    pos = np.array([0, 3, 7, 8, 2000])
    y = orc.rope_rotate(x, pos)
    assert np.array_equal(y[0], x[0])
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-13)
    assert np.allclose(orc.rope_rotate(y, pos, inverse=True), x, atol=1e-13)
    with pytest.raises(ValueError):
        orc.rope_rotate(np.zeros((2, 1, 3)), [0, 1])


def test_scores_depend_on_the_position_difference_only():
    rng = np.random.default_rng(2)
    q, k = rng.normal(size=(1, 1, 32)), rng.normal(size=(1, 1, 32))
    s0 = (orc.rope_rotate(q, [17]) * orc.rope_rotate(k, [5])).sum()
    s1 = (orc.rope_rotate(q, [1017]) * orc.rope_rotate(k, [1005])).sum()
    s2 = (orc.rope_rotate(q, [18]) * orc.rope_rotate(k, [5])).sum()
    assert abs(s0 - s1) <= 1e-10 and abs(s0 - s2) > 1e-3


def _case(B=2, S=12, D=16, H=4, G=2, seed=3):
    rng = np.random.default_rng(seed)
    d = D // H
    c = dict(xq=rng.normal(size=(B, S, D)), xkv=rng.normal(size=(B, S, D)), wq=rng.normal(size=(D, H * d)) * 0.4,
             wk=rng.normal(size=(D, G * d)) * 0.4, wv=rng.normal(size=(D, G * d)) * 0.4,
             wo=rng.normal(size=(H * d, D)) * 0.4)
    return c, dict(n_q_heads=H, n_kv_heads=G), rng.normal(size=(B, S, D))


def test_shifting_all_positions_changes_nothing_and_rope_changes_something():
    c, kw, _ = _case()
    mask = orc.dense_mask(12, 12, 3, 1)
    a = orc.xattn_forward(**c, **kw, mask=mask, rope=dict(base=500.0))
    b = orc.xattn_forward(**c, **kw, mask=mask, rope=dict(base=500.0, q_pos=np.arange(12) + 40, k_pos=np.arange(12) + 40))
    assert np.allclose(a["y"], b["y"], atol=1e-11) and np.allclose(a["lse"][np.isfinite(a["lse"])], b["lse"][np.isfinite(b["lse"])], atol=1e-11)
    plain = orc.xattn_forward(**c, **kw, mask=mask)
    assert not np.allclose(a["y"], plain["y"], atol=1e-3)
    assert np.array_equal(a["v"], plain["v"])                                  # V is not rotated
    assert np.array_equal(a["q"][:, 0], plain["q"][:, 0])                      # position 0: identity


def _torch_rope(x, pos, base):                                                 # rotate-half form used by the LLaMA family
    d = x.shape[-1]
    inv = base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.tensor(pos, dtype=torch.float64)[:, None] * inv[None, :]
    emb = torch.cat([ang, ang], dim=-1)
    cos, sin = emb.cos()[:, None, :], emb.sin()[:, None, :]
    rot = torch.cat([-x[..., d // 2:], x[..., :d // 2]], dim=-1)
    return x * cos + rot * sin


def test_forward_and_gradients_against_torch_autograd():
    c, kw, dy = _case()
    H, G = kw["n_q_heads"], kw["n_kv_heads"]
    B, S, D = c["xq"].shape
    d = c["wq"].shape[1] // H
    base = 777.0
    t = {n: torch.tensor(v, dtype=torch.float64, requires_grad=True) for n, v in c.items()}
    pos = list(range(S))
    q = _torch_rope((t["xq"] @ t["wq"]).view(B, S, H, d), pos, base).transpose(1, 2)
    k = _torch_rope((t["xkv"] @ t["wk"]).view(B, S, G, d), pos, base).transpose(1, 2).repeat_interleave(H // G, dim=1)
    v = (t["xkv"] @ t["wv"]).view(B, S, G, d).transpose(1, 2).repeat_interleave(H // G, dim=1)
    mask = torch.tensor(orc.dense_mask_loops(S, S, 3, 1))
    sees = mask.any(dim=1)
    nb = int((~sees).sum())
    o = torch.nn.functional.scaled_dot_product_attention(q[:, :, sees], k, v, attn_mask=mask[sees])
    o = torch.cat([torch.zeros(B, H, nb, d, dtype=torch.float64), o], dim=2)
    y = o.transpose(1, 2).reshape(B, S, H * d) @ t["wo"]
    (y * torch.tensor(dy)).sum().backward()
    g = orc.xattn_backward(dy, **c, **kw, mask=mask.numpy(), rope=dict(base=base))
    assert np.allclose(g["y"], y.detach().numpy(), atol=1e-12)
    for n, gn in (("xq", "dxq"), ("xkv", "dxkv"), ("wq", "dwq"), ("wk", "dwk"), ("wv", "dwv"), ("wo", "dwo")):
        assert np.allclose(g[gn], t[n].grad.numpy(), atol=1e-11), gn


def test_decode_with_rotated_cache_reproduces_the_training_row():
    """k = 1: query p of the training forward sees keys j < p; the draft step over a cache appended with rotated
    keys, with the query rotated to position p, gives the same row."""
    c, kw, _ = _case(B=1, S=10)
    rope = dict(base=300.0)
    fw = orc.xattn_forward(**c, **kw, mask=orc.dense_mask(10, 10, 1, 0), rope=rope)
    G, d = kw["n_kv_heads"], fw["k"].shape[-1]
    kc, vc = np.zeros((10, G, d)), np.zeros((10, G, d))
    kc, vc = orc.kv_append(kc, vc, 0, c["xkv"][0, :6], c["wk"], c["wv"], n_kv_heads=G, rope=dict(base=300.0, k_pos=np.arange(6)))
    kc, vc = orc.kv_append(kc, vc, 6, c["xkv"][0, 6:], c["wk"], c["wv"], n_kv_heads=G, rope=dict(base=300.0, k_pos=np.arange(6, 10)))
    assert np.allclose(kc, fw["k"][0], atol=1e-13)
    p = 7
    ds = orc.draft_step(c["xq"][0, p:p + 1], kc[:p], vc[:p], c["wq"], c["wo"], **kw, rope=dict(base=300.0, q_pos=[p]))
    assert np.allclose(ds["y"][0], fw["y"][0, p], atol=1e-12)
    tr = orc.draft_step_tree(c["xq"][0, p:p + 1], kc[:p], vc[:p], c["wq"], c["wo"], n_true=p, tree_mask=np.zeros((1, 0), bool),
                             **kw, rope=dict(base=300.0, q_pos=[p]))
    assert np.allclose(tr["y"], ds["y"], atol=1e-14)


def test_simulation_step_places_predicted_keys_at_their_own_positions():
    """With rope, the simulation step equals the plain masked forward over the concatenated keys whose second half
    carries positions 0..L-1 again; t = 0 is the early stage with rope."""
    c, kw, dy = _case()
    xp = np.random.default_rng(9).normal(size=c["xkv"].shape)
    rope = dict(base=250.0)
    a = orc.xattn_backward_sim(dy, c["xq"], c["xkv"], xp, c["wq"], c["wk"], c["wv"], c["wo"], **kw, k=4, eps=1, t=0, rope=rope)
    b = orc.xattn_backward(dy, **c, **kw, mask=orc.dense_mask(12, 12, 4, 1), rope=rope)
    for n in ("y", "dxq", "dxkv", "dwq", "dwk"):
        assert np.allclose(a[n], b[n], atol=1e-12), n
    f = orc.xattn_forward_sim(c["xq"], c["xkv"], xp, c["wq"], c["wk"], c["wv"], c["wo"], **kw, k=4, eps=1, t=2, rope=rope)
    kp_plain = (xp @ c["wk"]).reshape(2, 12, 2, -1)
    assert np.allclose(f["kp"], orc.rope_rotate(kp_plain, np.arange(12), 250.0), atol=1e-13)
