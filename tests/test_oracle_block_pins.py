"""Pins of the draft-block oracle (CPU only; section 4.1, Eq. 1): RMSNorm and the
gated feed-forward against torch's float64 library routines and autograd,
closed forms and invariants, the two residual lines of Eq. 1 in special
cases, the whole block against an independent torch construction, finite
differences."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import beagle_oracle as orc
from oracle import block_oracle as blk

T64 = torch.float64


def _t(a, grad=False):
    return torch.tensor(np.asarray(a, np.float64), dtype=T64, requires_grad=grad)


# ------------------------------------------------------------------ RMSNorm
@pytest.mark.parametrize("eps", [0.0, 1e-5, 0.3])
def test_rmsnorm_equals_the_library_routine(eps):
    rng = np.random.default_rng(0)
    x, g = rng.normal(size=(3, 5, 16)) * 3, rng.normal(size=16)
    want = F.rms_norm(_t(x), (16,), _t(g), eps).numpy()
    assert np.allclose(blk.rmsnorm(x, g, eps), want, rtol=1e-13, atol=1e-13)


def test_rmsnorm_invariants():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(7, 32))
    one = np.ones(32)
    out = blk.rmsnorm(x, one, 0.0)
    assert np.allclose(np.sqrt((out ** 2).mean(-1)), 1.0, atol=1e-14)          # unit RMS
    assert np.allclose(blk.rmsnorm(5.0 * x, one, 0.0), out, atol=1e-14)         # scale invariance at eps = 0
    assert np.array_equal(blk.rmsnorm(x, None, 1e-5), x)                        # no gain: identity
    g = rng.normal(size=32)
    assert np.allclose(blk.rmsnorm(x, g, 0.0), out * g, atol=1e-14)             # the gain is a plain factor
    # a constant row of value c with eps: c / sqrt(c^2 + eps)
    assert np.allclose(blk.rmsnorm(np.full((1, 8), 2.0), np.ones(8), 5.0), 2.0 / 3.0)


def test_rmsnorm_backward_autograd_finite_differences_and_orthogonality():
    rng = np.random.default_rng(2)
    x, g, dout = rng.normal(size=(4, 6, 12)), rng.normal(size=12), rng.normal(size=(4, 6, 12))
    eps = 1e-3
    xt, gt = _t(x, True), _t(g, True)
    (F.rms_norm(xt, (12,), gt, eps) * _t(dout)).sum().backward()
    dx, dg = blk.rmsnorm_backward(dout, x, g, eps)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12) and np.allclose(dg, gt.grad.numpy(), atol=1e-12)
    loss = lambda xx, gg: float((blk.rmsnorm(xx, gg, eps) * dout).sum())
    d = rng.normal(size=x.shape)
    fd = (loss(x + 1e-6 * d, g) - loss(x - 1e-6 * d, g)) / 2e-6
    assert abs(fd - (dx * d).sum()) <= 1e-6 * max(1.0, abs(fd))
    # at eps = 0 the output does not change along x itself: <x, dx> = 0 for every row
    dx0, _ = blk.rmsnorm_backward(dout, x, g, 0.0)
    assert np.abs((dx0 * x).sum(-1)).max() <= 1e-12
    assert blk.rmsnorm_backward(dout, x, None, eps)[1] is None
    assert np.array_equal(blk.rmsnorm_backward(dout, x, None, eps)[0], dout)


# ------------------------------------------------------------------ feed-forward
def test_silu_closed_forms():
    I = np.eye(3)
    u = np.array([[0.0, 2.0, -2.0]])
    f = blk.mlp_forward(u, I, np.ones((3, 3)) * 0 + I, I)        # gate = up = z, down = identity
    # silu(0) = 0; silu(u) - silu(-u) = u
    silu = f["m"] / np.where(u == 0, 1, u)
    assert silu[0, 0] == 0.0
    assert np.isclose(silu[0, 1] - silu[0, 2], 2.0, atol=1e-15)
    assert np.isclose(silu[0, 1], 2.0 / (1.0 + np.exp(-2.0)))
    # derivative of silu at 0 is 1/2: finite difference through the MLP with up = 1
    h = 1e-6
    a = blk.mlp_forward(np.array([[h]]), np.ones((1, 1)), np.zeros((1, 1)), np.ones((1, 1)))
    assert a["out"][0, 0] == 0.0                                  # up = 0 -> nothing passes the gate
    m = lambda v: float(blk.mlp_forward(np.array([[v, 1.0]]), np.array([[1.0], [0.0]]), np.array([[0.0], [1.0]]),
                                        np.ones((1, 1)))["out"][0, 0])
    assert abs((m(h) - m(-h)) / (2 * h) - 0.5) <= 1e-9


def test_mlp_equals_torch_and_autograd():
    rng = np.random.default_rng(3)
    z, dout = rng.normal(size=(2, 5, 8)), rng.normal(size=(2, 5, 8))
    wg, wu, wd = rng.normal(size=(8, 12)) * 0.5, rng.normal(size=(8, 12)) * 0.5, rng.normal(size=(12, 8)) * 0.5
    zt, a, b, c = _t(z, True), _t(wg, True), _t(wu, True), _t(wd, True)
    out = (F.silu(zt @ a) * (zt @ b)) @ c
    assert np.allclose(blk.mlp_forward(z, wg, wu, wd)["out"], out.detach().numpy(), atol=1e-13)
    (out * _t(dout)).sum().backward()
    g = blk.mlp_backward(dout, z, wg, wu, wd)
    for n, t in (("dz", zt), ("dw_gate", a), ("dw_up", b), ("dw_down", c)):
        assert np.allclose(g[n], t.grad.numpy(), atol=1e-12), n
    # swapping gate and up changes the result (they are not symmetric)
    assert not np.allclose(blk.mlp_forward(z, wu, wg, wd)["out"], out.detach().numpy())


# ------------------------------------------------------------------ the block
def _case(seed=4, B=2, S=11, D=8, H=2, G=1, Fdim=12, gains=True):
    rng = np.random.default_rng(seed)
    d = D // H
    c = dict(e=rng.normal(size=(B, S, D)), hs=rng.normal(size=(B, S, D)) * 2,
             wq=rng.normal(size=(D, H * d)) * 0.4, wk=rng.normal(size=(D, G * d)) * 0.4,
             wv=rng.normal(size=(D, G * d)) * 0.4, wo=rng.normal(size=(H * d, D)) * 0.4,
             w_gate=rng.normal(size=(D, Fdim)) * 0.4, w_up=rng.normal(size=(D, Fdim)) * 0.4,
             w_down=rng.normal(size=(Fdim, D)) * 0.4)
    kw = dict(n_q_heads=H, n_kv_heads=G, k=3, eps=1, rms_eps=1e-4)
    if gains:
        kw.update(g_q=1 + 0.3 * rng.normal(size=D), g_kv=1 + 0.3 * rng.normal(size=D), g_mlp=1 + 0.3 * rng.normal(size=D))
    return c, kw, rng.normal(size=(B, S, D))


def test_the_two_residual_lines_of_eq1():
    c, kw, _ = _case(gains=False)
    # no normalisation, W_down = 0: h = y = CrossAttn + e
    c0 = dict(c, w_down=np.zeros_like(c["w_down"]))
    f = blk.block_forward(**c0, **kw)
    mask = orc.dense_mask(11, 11, 3, 1)
    att = orc.xattn_forward(c["e"], c["hs"], c["wq"], c["wk"], c["wv"], c["wo"], n_q_heads=2, n_kv_heads=1, mask=mask)["y"]
    assert np.array_equal(f["h"], f["y"]) and np.allclose(f["y"], att + c["e"], atol=1e-15)
    # Wo = 0: y = e and h - e = MLP(e)
    f = blk.block_forward(**dict(c, wo=np.zeros_like(c["wo"])), **kw)
    assert np.array_equal(f["y"], c["e"])
    assert np.allclose(f["h"] - c["e"], blk.mlp_forward(c["e"], c["w_gate"], c["w_up"], c["w_down"])["out"], atol=1e-14)
    # blind queries (first window): y = e exactly
    f = blk.block_forward(**c, **kw)
    blind = ~mask.any(axis=1)
    assert blind.any() and np.array_equal(f["y"][:, blind], c["e"][:, blind])


def _torch_block(c, kw, leaves):
    """The same block from torch primitives (library RMSNorm, SDPA with a boolean mask on the rows that see
    something, library SiLU)."""
    t = {n: _t(v, n in leaves or leaves == "all") for n, v in c.items()}
    gains = {n: (_t(kw[n], True) if kw.get(n) is not None else None) for n in ("g_q", "g_kv", "g_mlp")}
    H, G = kw["n_q_heads"], kw["n_kv_heads"]
    B, S, D = c["e"].shape
    L = c["hs"].shape[1]
    d = c["wq"].shape[1] // H
    norm = lambda x, g: x if g is None else F.rms_norm(x, (D,), g, kw["rms_eps"])
    xq, xkv = norm(t["e"], gains["g_q"]), norm(t["hs"], gains["g_kv"])
    q = (xq @ t["wq"]).view(B, S, H, d).transpose(1, 2)
    k = (xkv @ t["wk"]).view(B, L, G, d).transpose(1, 2).repeat_interleave(H // G, dim=1)
    v = (xkv @ t["wv"]).view(B, L, G, d).transpose(1, 2).repeat_interleave(H // G, dim=1)
    mask = torch.tensor(orc.dense_mask_loops(S, L, kw["k"], kw["eps"]))
    sees = mask.any(dim=1)
    o_seen = F.scaled_dot_product_attention(q[:, :, sees], k, v, attn_mask=mask[sees])
    nb = int((~sees).sum())
    assert not sees[:nb].any() and sees[nb:].all()                # the blind queries are the first ones
    o = torch.cat([torch.zeros(B, H, nb, d, dtype=T64), o_seen], dim=2)
    y = o.transpose(1, 2).reshape(B, S, H * d) @ t["wo"] + t["e"]
    z = norm(y, gains["g_mlp"])
    h = (F.silu(z @ t["w_gate"]) * (z @ t["w_up"])) @ t["w_down"] + y
    return h, t, gains


@pytest.mark.parametrize("gains", [True, False])
def test_block_forward_and_all_gradients_against_torch(gains):
    c, kw, dh = _case(gains=gains)
    h, t, g = _torch_block(c, kw, "all")
    f = blk.block_forward(**c, **kw)
    assert np.allclose(f["h"], h.detach().numpy(), atol=1e-12)
    (h * _t(dh)).sum().backward()
    b = blk.block_backward(dh, **c, **kw)
    names = dict(de="e", dhs="hs", dwq="wq", dwk="wk", dwv="wv", dwo="wo", dw_gate="w_gate", dw_up="w_up", dw_down="w_down")
    for gn, n in names.items():
        assert np.allclose(b[gn], t[n].grad.numpy(), atol=1e-11), gn
    for n in ("g_q", "g_kv", "g_mlp"):
        if gains:
            assert np.allclose(b["d" + n], g[n].grad.numpy(), atol=1e-11), n
        else:
            assert b["d" + n] is None


def test_block_gradients_by_finite_differences():
    c, kw, dh = _case(seed=6)
    b = blk.block_backward(dh, **c, **kw)
    rng = np.random.default_rng(7)
    names = dict(e="de", hs="dhs", wq="dwq", wk="dwk", wv="dwv", wo="dwo", w_gate="dw_gate", w_up="dw_up", w_down="dw_down")
    loss = lambda cc, kk: float((blk.block_forward(**cc, **kk)["h"] * dh).sum())
    for n, gn in names.items():
        d = rng.normal(size=c[n].shape)
        fd = (loss(dict(c, **{n: c[n] + 1e-6 * d}), kw) - loss(dict(c, **{n: c[n] - 1e-6 * d}), kw)) / 2e-6
        assert abs(fd - (b[gn] * d).sum()) <= 2e-6 * max(1.0, abs(fd)), n
    for n in ("g_q", "g_kv", "g_mlp"):
        d = rng.normal(size=kw[n].shape)
        fd = (loss(c, dict(kw, **{n: kw[n] + 1e-6 * d})) - loss(c, dict(kw, **{n: kw[n] - 1e-6 * d}))) / 2e-6
        assert abs(fd - (b["d" + n] * d).sum()) <= 2e-6 * max(1.0, abs(fd)), n


# ------------------------------------------------------------------ the block at decode time
@pytest.mark.parametrize("gains,rope", [(True, None), (False, None), (True, dict(base=100.0))])
def test_block_draft_step_reproduces_the_training_block_row(gains, rope):
    """k = 1: row p of the training block sees keys j < p.  The decode-time block over a cache holding the K/V rows of
    the (normalised) states 0 .. p-1, fed with embedding p, gives the same h (the training block is pinned above)."""
    c, kw, _ = _case(B=1, S=9, gains=gains)
    kw = dict(kw, k=1, eps=0)
    f = blk.block_forward(**c, **kw, rope=rope)
    G = kw["n_kv_heads"]
    kc, vc = f["attn"]["k"][0], f["attn"]["v"][0]             # rows as the training forward projected (and rotated) them
    for p in (1, 4, 8):
        dkw = dict(g_q=kw.get("g_q"), g_mlp=kw.get("g_mlp"), rms_eps=kw["rms_eps"], n_q_heads=kw["n_q_heads"], n_kv_heads=G)
        r = None if rope is None else dict(rope, q_pos=[p])
        d = blk.block_draft_step(c["e"][0, p:p + 1], kc[:p], vc[:p], c["wq"], c["wo"], c["w_gate"], c["w_up"], c["w_down"],
                                 **dkw, rope=r)
        assert np.allclose(d["h"][0], f["h"][0, p], atol=1e-12), p
        assert np.allclose(d["y"][0], f["y"][0, p], atol=1e-12), p
    # drafted rows under a tree: hiding a drafted row equals dropping it from the cache
    p = 6
    tm = np.array([[True, False]])
    a = blk.block_draft_step(c["e"][0, p:p + 1], kc[:p], vc[:p], c["wq"], c["wo"], c["w_gate"], c["w_up"], c["w_down"],
                             **dkw, n_true=p - 2, tree_mask=tm)
    b = blk.block_draft_step(c["e"][0, p:p + 1], kc[:p - 1], vc[:p - 1], c["wq"], c["wo"], c["w_gate"], c["w_up"], c["w_down"], **dkw)
    assert np.allclose(a["h"], b["h"], atol=1e-13)


# ------------------------------------------------------------------ the block in a late-stage simulation step
def test_block_simulation_step_zero_is_the_plain_block_and_gradients_check():
    c, kw, dh = _case(seed=8)
    xp = np.random.default_rng(11).normal(size=c["hs"].shape) * 3
    a = blk.block_backward(dh, **c, **kw, xpred=xp, t=0)
    b = blk.block_backward(dh, **c, **kw)
    for n in ("de", "dhs", "dwq", "dwk", "dw_gate", "dg_q", "dg_kv", "dg_mlp"):
        assert np.allclose(a[n], b[n], atol=1e-12), n
    assert np.allclose(a["fwd"]["h"], b["fwd"]["h"], atol=1e-13) and not a["dxpred"].any()
    # t = 2: something changes, and every gradient agrees with finite differences (xpred and g_kv included:
    # the gain sees both key/value sources)
    g = blk.block_backward(dh, **c, **kw, xpred=xp, t=2)
    assert not np.allclose(g["fwd"]["h"], b["fwd"]["h"], atol=1e-6) and g["dxpred"].any()
    rng = np.random.default_rng(12)
    loss = lambda cc, kk, x: float((blk.block_forward(**cc, **kk, xpred=x, t=2)["h"] * dh).sum())
    for n, gn in (("e", "de"), ("hs", "dhs"), ("wk", "dwk"), ("wv", "dwv"), ("w_up", "dw_up")):
        d = rng.normal(size=c[n].shape)
        fd = (loss(dict(c, **{n: c[n] + 1e-6 * d}), kw, xp) - loss(dict(c, **{n: c[n] - 1e-6 * d}), kw, xp)) / 2e-6
        assert abs(fd - (g[gn] * d).sum()) <= 2e-6 * max(1.0, abs(fd)), n
    d = rng.normal(size=xp.shape)
    fd = (loss(c, kw, xp + 1e-6 * d) - loss(c, kw, xp - 1e-6 * d)) / 2e-6
    assert abs(fd - (g["dxpred"] * d).sum()) <= 2e-6 * max(1.0, abs(fd))
    d = rng.normal(size=kw["g_kv"].shape)
    fd = (loss(c, dict(kw, g_kv=kw["g_kv"] + 1e-6 * d), xp) - loss(c, dict(kw, g_kv=kw["g_kv"] - 1e-6 * d), xp)) / 2e-6
    assert abs(fd - (g["dg_kv"] * d).sum()) <= 2e-6 * max(1.0, abs(fd))
    # the predicted states pass through the key/value normalisation: scaling them changes nothing at rms_eps = 0
    kw0 = dict(kw, rms_eps=0.0)
    h1 = blk.block_forward(**c, **kw0, xpred=xp, t=2)["h"]
    h2 = blk.block_forward(**c, **kw0, xpred=7.0 * xp, t=2)["h"]
    assert np.allclose(h1, h2, atol=1e-12)


def test_block_kv_append_builds_the_rows_the_training_block_uses():
    c, kw, _ = _case(B=1, S=9)
    f = blk.block_forward(**c, **dict(kw, k=1, eps=0), rope=dict(base=50.0))
    G = kw["n_kv_heads"]
    d = f["attn"]["k"].shape[-1]
    kc, vc = np.zeros((9, G, d)), np.zeros((9, G, d))
    kc, vc = blk.block_kv_append(kc, vc, 0, c["hs"][0, :5], c["wk"], c["wv"], g_kv=kw["g_kv"], rms_eps=kw["rms_eps"],
                                 n_kv_heads=G, rope=dict(base=50.0, k_pos=np.arange(5)))
    kc, vc = blk.block_kv_append(kc, vc, 5, c["hs"][0, 5:], c["wk"], c["wv"], g_kv=kw["g_kv"], rms_eps=kw["rms_eps"],
                                 n_kv_heads=G, rope=dict(base=50.0, k_pos=np.arange(5, 9)))
    assert np.allclose(kc, f["attn"]["k"][0], atol=1e-13) and np.allclose(vc, f["attn"]["v"][0], atol=1e-13)
    # without the gain it is the plain append
    a = blk.block_kv_append(kc, vc, 2, c["hs"][0, :3], c["wk"], c["wv"], n_kv_heads=G)
    b = orc.kv_append(kc, vc, 2, c["hs"][0, :3], c["wk"], c["wv"], n_kv_heads=G)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
