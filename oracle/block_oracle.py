"""Float64 CPU oracle for the whole single-layer draft block around the
cross-attention (paper section 4.1, Eq. 1):

    y_n = CrossAttn(h_{1:n-1}, e(t_n)) + e(t_n)
    h_n = MLP(y_n) + y_n

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
CPU-baseline leg of the benchmark; shares no code with the HIP path.

Eq. 1 fixes the two residual connections and says that the MLP is a
point-wise feed-forward layer; it leaves out normalisation and the MLP's form
on purpose ("layer details omitted").  Readings taken here, all PARITY
UNPINNED by the paper beyond Eq. 1:
  * the block follows the pre-normalisation layout of the LLaMA / Vicuna
    targets the drafts are trained for: every sublayer reads an RMS-normalised
    copy of its input, and each residual adds the UN-normalised stream;
  * RMSNorm(x) = x / sqrt(mean_c(x_c^2) + rms_eps) * gain, one gain vector per
    normalised input: g_q for the token embeddings e (the queries' source),
    g_kv for the key/value states, g_mlp for y.  A gain of None switches that
    normalisation off (identity), which gives Eq. 1 exactly as printed;
  * the MLP is the gated SiLU feed-forward of those targets, no biases:
        MLP(z) = ( silu(z W_gate) * (z W_up) ) W_down,  silu(u) = u * sigmoid(u),
    with W_gate, W_up [D, F] and W_down [F, D] stored [in, out];
  * the mask, scale and head conventions are those of beagle_oracle.

Everything is written as the plain definition: dense matrices, no fusion, the
backward is the chain rule term by term.
"""
from __future__ import annotations

import numpy as np

from oracle import beagle_oracle as orc

F64 = np.float64


# --------------------------------------------------------------------------
# RMSNorm
# --------------------------------------------------------------------------
def rmsnorm(x, gain, rms_eps):
    """x [..., D] -> x / sqrt(mean(x^2) + rms_eps) * gain; gain None: identity."""
    x = np.asarray(x, F64)
    if gain is None:
        return x.copy()
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + rms_eps)
    return x * r * np.asarray(gain, F64)


def rmsnorm_backward(dout, x, gain, rms_eps):
    """Gradients of sum(dout * rmsnorm(x)) w.r.t. x and gain.
    With r = (mean(x^2) + eps)^(-1/2) and xh = x r:
        d xh = dout * gain
        dx   = r * (d xh - xh * mean_c(d xh * xh))      (derivative of r through x)
        dgain = sum over rows of dout * xh
    gain None: (dout, None)."""
    dout, x = np.asarray(dout, F64), np.asarray(x, F64)
    if gain is None:
        return dout.copy(), None
    gain = np.asarray(gain, F64)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + rms_eps)
    xh = x * r
    dxh = dout * gain
    dx = r * (dxh - xh * np.mean(dxh * xh, axis=-1, keepdims=True))
    dgain = (dout * xh).reshape(-1, x.shape[-1]).sum(axis=0)
    return dx, dgain


# --------------------------------------------------------------------------
# Gated SiLU feed-forward
# --------------------------------------------------------------------------
def _sigmoid(u):
    return 1.0 / (1.0 + np.exp(-u))


def mlp_forward(z, w_gate, w_up, w_down):
    """Returns dict: u = z W_gate, w = z W_up, m = silu(u) * w, out = m W_down."""
    z = np.asarray(z, F64)
    w_gate, w_up, w_down = (np.asarray(a, F64) for a in (w_gate, w_up, w_down))
    u = z @ w_gate
    w = z @ w_up
    m = u * _sigmoid(u) * w
    return dict(u=u, w=w, m=m, out=m @ w_down)


def mlp_backward(dout, z, w_gate, w_up, w_down):
    """Gradients of sum(dout * MLP(z)): dz, dw_gate, dw_up, dw_down.
    d silu(u)/du = sig(u) * (1 + u * (1 - sig(u)))."""
    dout, z = np.asarray(dout, F64), np.asarray(z, F64)
    w_gate, w_up, w_down = (np.asarray(a, F64) for a in (w_gate, w_up, w_down))
    f = mlp_forward(z, w_gate, w_up, w_down)
    u, w, m = f["u"], f["w"], f["m"]
    D, F = w_gate.shape
    z2, dout2 = z.reshape(-1, D), dout.reshape(-1, D)
    dm = dout @ w_down.T
    sg = _sigmoid(u)
    du = dm * w * sg * (1.0 + u * (1.0 - sg))
    dw = dm * u * sg
    dz = du @ w_gate.T + dw @ w_up.T
    return dict(dz=dz, dw_gate=z2.T @ du.reshape(-1, F), dw_up=z2.T @ dw.reshape(-1, F),
                dw_down=m.reshape(-1, F).T @ dout2, du=du, dw=dw, dm=dm)


# --------------------------------------------------------------------------
# The block (Eq. 1)
# --------------------------------------------------------------------------
def block_forward(e, hs, wq, wk, wv, wo, w_gate, w_up, w_down, *, g_q=None, g_kv=None, g_mlp=None,
                  rms_eps=1e-5, n_q_heads, n_kv_heads, k, eps=0, scale=None, rope=None, xpred=None, t=0):
    """e [B,S,D] token embeddings, hs [B,L,D] key/value states.  Returns dict with
    h [B,S,D] (the block's output), y (after the first residual), the normalised
    inputs xq, xkv, z, the attention's own results (attn: the dict of
    xattn_forward) and the MLP's (mlp).
    xpred [B,L,D], t: late-stage simulation step t (section 4.2, second half) --
    the attention is beagle_oracle.xattn_forward_sim; the predicted states are
    key/value source states like hs (they are this block's own earlier outputs
    h), so they pass through the same normalisation g_kv (xp in the result)."""
    e, hs = np.asarray(e, F64), np.asarray(hs, F64)
    xq = rmsnorm(e, g_q, rms_eps)
    xkv = rmsnorm(hs, g_kv, rms_eps)
    mask = orc.dense_mask(e.shape[1], hs.shape[1], k, eps)
    if xpred is not None:
        xp = rmsnorm(xpred, g_kv, rms_eps)
        attn = orc.xattn_forward_sim(xq, xkv, xp, wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, k=k,
                                     eps=eps, t=t, scale=scale, rope=rope)
        y = attn["y"] + e
        z = rmsnorm(y, g_mlp, rms_eps)
        mlp = mlp_forward(z, w_gate, w_up, w_down)
        return dict(h=mlp["out"] + y, y=y, xq=xq, xkv=xkv, xp=xp, z=z, attn=attn, mlp=mlp, mask=mask)
    attn = orc.xattn_forward(xq, xkv, wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, mask=mask,
                             scale=scale, rope=rope)
    y = attn["y"] + e                                   # Eq. 1, second line
    z = rmsnorm(y, g_mlp, rms_eps)
    mlp = mlp_forward(z, w_gate, w_up, w_down)
    h = mlp["out"] + y                                  # Eq. 1, first line
    return dict(h=h, y=y, xq=xq, xkv=xkv, z=z, attn=attn, mlp=mlp, mask=mask)


def block_backward(dh, e, hs, wq, wk, wv, wo, w_gate, w_up, w_down, *, g_q=None, g_kv=None, g_mlp=None,
                   rms_eps=1e-5, n_q_heads, n_kv_heads, k, eps=0, scale=None, rope=None, xpred=None, t=0):
    """Gradients of sum(dh * h) w.r.t. every input of block_forward: de, dhs, the
    seven weight matrices and the three gains (None where the gain is None); with
    xpred also dxpred, and g_kv's gradient collects both key/value sources."""
    dh = np.asarray(dh, F64)
    f = block_forward(e, hs, wq, wk, wv, wo, w_gate, w_up, w_down, g_q=g_q, g_kv=g_kv, g_mlp=g_mlp,
                      rms_eps=rms_eps, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, k=k, eps=eps, scale=scale, rope=rope,
                      xpred=xpred, t=t)
    if xpred is not None:
        mb = mlp_backward(dh, f["z"], w_gate, w_up, w_down)
        dy_norm, dg_mlp = rmsnorm_backward(mb["dz"], f["y"], g_mlp, rms_eps)
        dy = dh + dy_norm
        ab = orc.xattn_backward_sim(dy, f["xq"], f["xkv"], f["xp"], wq, wk, wv, wo, n_q_heads=n_q_heads,
                                    n_kv_heads=n_kv_heads, k=k, eps=eps, t=t, scale=scale, rope=rope)
        de_norm, dg_q = rmsnorm_backward(ab["dxq"], e, g_q, rms_eps)
        dhs, dg_kv = rmsnorm_backward(ab["dxkv"], hs, g_kv, rms_eps)
        dxpred, dg_kv2 = rmsnorm_backward(ab["dxpred"], xpred, g_kv, rms_eps)
        return dict(de=dy + de_norm, dhs=dhs, dxpred=dxpred, dwq=ab["dwq"], dwk=ab["dwk"], dwv=ab["dwv"], dwo=ab["dwo"],
                    dw_gate=mb["dw_gate"], dw_up=mb["dw_up"], dw_down=mb["dw_down"], dg_q=dg_q,
                    dg_kv=None if g_kv is None else dg_kv + dg_kv2, dg_mlp=dg_mlp, dy=dy, fwd=f)
    # h = MLP(z) + y
    mb = mlp_backward(dh, f["z"], w_gate, w_up, w_down)
    dy_norm, dg_mlp = rmsnorm_backward(mb["dz"], f["y"], g_mlp, rms_eps)
    dy = dh + dy_norm
    # y = CrossAttn(xkv, xq) + e
    ab = orc.xattn_backward(dy, f["xq"], f["xkv"], wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                            mask=f["mask"], scale=scale, rope=rope)
    de_norm, dg_q = rmsnorm_backward(ab["dxq"], e, g_q, rms_eps)
    dhs, dg_kv = rmsnorm_backward(ab["dxkv"], hs, g_kv, rms_eps)
    return dict(de=dy + de_norm, dhs=dhs, dwq=ab["dwq"], dwk=ab["dwk"], dwv=ab["dwv"], dwo=ab["dwo"],
                dw_gate=mb["dw_gate"], dw_up=mb["dw_up"], dw_down=mb["dw_down"],
                dg_q=dg_q, dg_kv=dg_kv, dg_mlp=dg_mlp, dy=dy, fwd=f)


# --------------------------------------------------------------------------
# The block at decode time (section 4.1, last paragraphs: the same block decodes
# draft tokens autoregressively against cached K/V rows)
# --------------------------------------------------------------------------
def block_draft_step(x, k_cache, v_cache, wq, wo, w_gate, w_up, w_down, *, g_q=None, g_mlp=None, rms_eps=1e-5,
                     n_true=None, tree_mask=None, n_q_heads, n_kv_heads, scale=None, rope=None):
    """M draft token embeddings x [M, D] through Eq. 1 against a cache of already projected (and, with rope,
    already rotated) K/V rows: y = Attn(RMSNorm(x; g_q)) + x over the cache rows (all of them, or n_true true rows
    plus the drafted rows that tree_mask shows), h = MLP(RMSNorm(y; g_mlp)) + y.  Returns dict h, y, lse.
    The key/value side's normalisation (g_kv) and projections happened when the rows were appended."""
    x = np.asarray(x, F64)
    L = np.asarray(k_cache).shape[0]
    if n_true is None:
        n_true, tree_mask = L, np.zeros((x.shape[0], 0), bool)
    xn = rmsnorm(x, g_q, rms_eps)
    att = orc.draft_step_tree(xn, k_cache, v_cache, wq, wo, n_true=n_true, tree_mask=tree_mask, n_q_heads=n_q_heads,
                              n_kv_heads=n_kv_heads, scale=scale, rope=rope)
    y = att["y"] + x
    z = rmsnorm(y, g_mlp, rms_eps)
    h = mlp_forward(z, w_gate, w_up, w_down)["out"] + y
    return dict(h=h, y=y, lse=att["lse"])


def block_kv_append(k_cache, v_cache, pos, x_new, wk, wv, *, g_kv=None, rms_eps=1e-5, n_kv_heads, rope=None):
    """New cache rows for the block: the states (true ones from the target model, or drafted ones = earlier block
    outputs h) are key/value source states, so they take the key/value normalisation g_kv before the projections --
    exactly what block_forward does to hs.  Returns the updated copies of the caches."""
    return orc.kv_append(k_cache, v_cache, pos, rmsnorm(x_new, g_kv, rms_eps), wk, wv, n_kv_heads=n_kv_heads, rope=rope)
