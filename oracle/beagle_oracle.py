"""Float64 CPU oracle for Beagle's block-masked cross-attention.

TEST INFRASTRUCTURE ONLY.  This module is the slow, dense, obviously-correct
definition that the GPU path is compared against.  It is imported by the
tests, by the smoke check and by the CPU-baseline leg of the benchmark, and
by nothing else; it shares no code with the HIP path and never calls it.

What it computes (paper section 4.1, Eq. 2, with the early-stage mask of
section 4.2):

    Q = Xq Wq,  K = Xkv Wk,  V = Xkv Wv            per-head column slices
    s = softmax_j( <Q_i, K_j> / sqrt(d_h) )        over the VISIBLE keys only
    o_i = sum_j Mask_ij s_ij V_j
    y_i = [o^(1); ...; o^(H)] Wo

Everything is float64 NumPy on an explicit dense boolean mask.  No tiling, no
online softmax, no recomputation: the backward pass is the chain rule written
on the stored dense probability matrix.

Readings of the paper taken here (the paper is silent or ambiguous):
  * The mask is applied BEFORE normalisation (masked scores are -inf), so that
    visible weights sum to one and masked weights are exactly zero.  Eq. 2
    read literally multiplies the mask after the softmax.
  * One mask for every head and batch entry.
  * Windows tile the whole sequence: starts are eps + w*k for every integer w
    whose window touches the sequence, including the partial leading window
    when eps > 0.
  * A query that sees no key gets a zero output row, LSE = -inf, and
    contributes no gradient.  PARITY UNPINNED by the paper: this is a
    convention (the paper never discusses the empty softmax).
  * GQA: query head h reads KV head h // (H // G).
  * Weights are stored [in, out]; scale defaults to 1/sqrt(d_h) (Eq. 2).
  * LSE is the natural-log log-sum-exp of the scaled visible scores.

Indices are 0-based here; the paper is 1-based.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Mask (section 4.1 "diagonal scores are also masked"; section 4.2 windows)
# --------------------------------------------------------------------------
def _window_starts(seq_q: int, k: int, eps: int):
    """Window starts eps + w*k (section 4.2) for every window that overlaps
    queries 0 .. seq_q-1, the partial leading one (start eps-k < 0) included."""
    if k < 1 or not (0 <= eps < k):
        raise ValueError("need k >= 1 and 0 <= eps < k")
    n = eps - k if eps > 0 else 0
    starts = []
    while n < seq_q:
        starts.append(n)
        n += k
    return starts


def dense_mask_loops(seq_q: int, seq_kv: int, k: int, eps: int = 0) -> np.ndarray:
    """Boolean [seq_q, seq_kv]; True where query p may attend key j.

    Element-by-element from the two prose rules (small sizes only):
      (1) strict causality: key j is hidden from query p when j >= p
          (section 4.1: the diagonal is masked too);
      (2) a window that starts at n (0-based) holds queries n .. n+k-1 and
          hides keys n .. n+k-1 from each of them (section 4.2).
    """
    m = np.ones((seq_q, seq_kv), dtype=bool)
    for p in range(seq_q):                       # rule (1)
        for j in range(seq_kv):
            if j >= p:
                m[p, j] = False
    for n in _window_starts(seq_q, k, eps):      # rule (2)
        for p in range(max(n, 0), min(n + k, seq_q)):
            for j in range(max(n, 0), min(n + k, seq_kv)):
                m[p, j] = False
    return m


def dense_mask(seq_q: int, seq_kv: int, k: int, eps: int = 0) -> np.ndarray:
    """Same mask as dense_mask_loops, with each rule applied as one array
    operation (rule 1: strictly-lower triangle; rule 2: one square block per
    window) so that full-size masks are affordable."""
    m = np.tri(seq_q, seq_kv, -1, dtype=bool)    # rule (1): j < p
    for n in _window_starts(seq_q, k, eps):      # rule (2)
        m[max(n, 0):min(n + k, seq_q), max(n, 0):min(n + k, seq_kv)] = False
    return m


def visible_counts(mask: np.ndarray) -> np.ndarray:
    """Number of visible keys per query row (int64 [seq_q])."""
    return mask.sum(axis=1).astype(np.int64)


# --------------------------------------------------------------------------
# Forward (Eq. 2)
# --------------------------------------------------------------------------
def _check_heads(H: int, G: int) -> int:
    if H < 1 or G < 1 or H % G:
        raise ValueError("n_kv_heads must divide n_q_heads")
    return H // G


def masked_softmax(scores: np.ndarray, mask: np.ndarray):
    """Row-wise softmax over visible entries.  Returns (P, LSE).

    Masked entries of P are exactly 0.0.  A row with no visible entry is all
    zero with LSE = -inf.
    """
    s = np.where(mask, scores, -np.inf)
    mx = s.max(axis=-1, keepdims=True)
    mx_safe = np.where(np.isfinite(mx), mx, 0.0)
    e = np.where(mask, np.exp(s - mx_safe), 0.0)
    l = e.sum(axis=-1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        P = np.where(l > 0, e / np.where(l > 0, l, 1.0), 0.0)
        lse = np.where(l > 0, mx_safe + np.log(np.where(l > 0, l, 1.0)), -np.inf)
    return P, lse[..., 0]


# --------------------------------------------------------------------------
# Rotary position embedding (optional).  Section 4.1 leaves positional
# embeddings out "for clarity"; the LLaMA / Vicuna targets the drafts are built
# for rotate queries and keys.  Reading taken here (PARITY UNPINNED by the
# paper): the rotate-half convention of those models -- channel c < d/2 is
# paired with channel c + d/2, angle = position * base^(-2c/d) -- applied to
# the projected Q at the query's sequence position and to the projected K at
# the key's sequence position, per head; V is not rotated.
# --------------------------------------------------------------------------
def rope_rotate(x, positions, base=10000.0, inverse=False):
    """x [..., P, heads, d] with d even, positions [P]: every (x_c, x_{c+d/2})
    pair is rotated by +angle (by -angle if inverse: the transpose, which is
    what the backward pass applies to gradients)."""
    x = np.asarray(x, F64)
    d = x.shape[-1]
    if d % 2:
        raise ValueError("rotary embedding needs an even head width")
    half = d // 2
    pos = np.asarray(positions, F64)
    if pos.shape != (x.shape[-3],):
        raise ValueError("one position per row")
    ang = pos[:, None] * (float(base) ** (-2.0 * np.arange(half) / d))[None, :]
    if inverse:
        ang = -ang
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def _rope_args(rope, n_q, n_k):
    """rope: None, or dict(base=..., q_pos=[n_q] or None, k_pos=[n_k] or None); default positions are the indices."""
    base = rope.get("base", 10000.0) or 10000.0
    q_pos = rope.get("q_pos")
    k_pos = rope.get("k_pos")
    return (base, np.arange(n_q) if q_pos is None else np.asarray(q_pos),
            np.arange(n_k) if k_pos is None else np.asarray(k_pos))


def xattn_forward(xq, xkv, wq, wk, wv, wo, *, n_q_heads, n_kv_heads, mask,
                  scale=None, keep_probs=False, rope=None):
    """Forward pass of Eq. 2 under an explicit dense mask.

    xq  [B, Sq, D]      draft-side query states e(t_i)
    xkv [B, L, D]       target hidden states h_j
    wq  [D, H*d]  wk, wv [D, G*d]  wo [H*d, D]
    mask bool [Sq, L]   shared by batch and heads
    rope: None, or dict(base, q_pos, k_pos) -- Q and K are rotated after the
    projections (rope_rotate); the returned q, k are the rotated ones.
    Returns dict: y [B,Sq,D], lse [B,H,Sq], q [B,Sq,H,d], k,v [B,L,G,d],
                  o [B,Sq,H,d] and, if keep_probs, p [B,H,Sq,L].
    """
    xq, xkv = np.asarray(xq, F64), np.asarray(xkv, F64)
    wq, wk, wv, wo = (np.asarray(w, F64) for w in (wq, wk, wv, wo))
    H, G = n_q_heads, n_kv_heads
    rep = _check_heads(H, G)
    B, Sq, D = xq.shape
    L = xkv.shape[1]
    d = wq.shape[1] // H
    if scale is None or scale == 0:
        scale = 1.0 / math.sqrt(d)
    mask = np.asarray(mask, bool)
    assert mask.shape == (Sq, L)

    q = (xq @ wq).reshape(B, Sq, H, d)
    k = (xkv @ wk).reshape(B, L, G, d)
    v = (xkv @ wv).reshape(B, L, G, d)
    if rope is not None:
        base, q_pos, k_pos = _rope_args(rope, Sq, L)
        q, k = rope_rotate(q, q_pos, base), rope_rotate(k, k_pos, base)
    o = np.zeros((B, Sq, H, d), F64)
    lse = np.zeros((B, H, Sq), F64)
    probs = np.zeros((B, H, Sq, L), F64) if keep_probs else None
    for b in range(B):
        for h in range(H):
            g = h // rep
            s = (q[b, :, h, :] @ k[b, :, g, :].T) * scale
            P, lse[b, h] = masked_softmax(s, mask)
            o[b, :, h, :] = P @ v[b, :, g, :]
            if keep_probs:
                probs[b, h] = P
    y = o.reshape(B, Sq, H * d) @ wo
    out = dict(y=y, lse=lse, q=q, k=k, v=v, o=o, scale=scale)
    if keep_probs:
        out["p"] = probs
    return out


# --------------------------------------------------------------------------
# Backward (chain rule of Eq. 2 on the dense probabilities)
# --------------------------------------------------------------------------
def xattn_backward(dy, xq, xkv, wq, wk, wv, wo, *, n_q_heads, n_kv_heads, mask,
                   scale=None, rope=None):
    """Gradients of sum(dy * y) with respect to every input of xattn_forward.

    Returns dict with dxq, dxkv, dwq, dwk, dwv, dwo and the intermediates
    dq [B,Sq,H,d], dk, dv [B,L,G,d], do [B,Sq,H,d], delta [B,H,Sq].
    """
    dy = np.asarray(dy, F64)
    xq, xkv = np.asarray(xq, F64), np.asarray(xkv, F64)
    wq, wk, wv, wo = (np.asarray(w, F64) for w in (wq, wk, wv, wo))
    H, G = n_q_heads, n_kv_heads
    rep = _check_heads(H, G)
    fw = xattn_forward(xq, xkv, wq, wk, wv, wo, n_q_heads=H, n_kv_heads=G,
                       mask=mask, scale=scale, keep_probs=False, rope=rope)
    q, k, v, o, scale = fw["q"], fw["k"], fw["v"], fw["o"], fw["scale"]
    B, Sq, D = xq.shape
    L = xkv.shape[1]
    d = q.shape[-1]
    mask = np.asarray(mask, bool)

    o2 = o.reshape(B * Sq, H * d)
    dy2 = dy.reshape(B * Sq, D)
    dwo = o2.T @ dy2
    do = (dy2 @ wo.T).reshape(B, Sq, H, d)

    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    delta = np.zeros((B, H, Sq), F64)
    for b in range(B):
        for h in range(H):
            g = h // rep
            s = (q[b, :, h, :] @ k[b, :, g, :].T) * scale
            P, _ = masked_softmax(s, mask)
            dO = do[b, :, h, :]
            dv[b, :, g, :] += P.T @ dO
            dP = dO @ v[b, :, g, :].T
            # softmax Jacobian: dS = P * (dP - sum_j P dP); the row sum equals
            # sum_c dO_c O_c because O = P V.
            dlt = (dO * o[b, :, h, :]).sum(axis=-1)
            delta[b, h] = dlt
            dS = P * (dP - dlt[:, None])
            dq[b, :, h, :] = (dS @ k[b, :, g, :]) * scale
            dk[b, :, g, :] += (dS.T @ q[b, :, h, :]) * scale

    if rope is not None:
        # dq, dk above are gradients of the ROTATED q, k; the rotation is orthogonal, so the gradients of the
        # projections' outputs are the same vectors rotated back
        base, q_pos, k_pos = _rope_args(rope, Sq, L)
        dq, dk = rope_rotate(dq, q_pos, base, inverse=True), rope_rotate(dk, k_pos, base, inverse=True)
    dq2 = dq.reshape(B * Sq, H * d)
    dk2 = dk.reshape(B * L, G * d)
    dv2 = dv.reshape(B * L, G * d)
    xq2 = xq.reshape(B * Sq, D)
    xkv2 = xkv.reshape(B * L, D)
    return dict(
        dxq=(dq2 @ wq.T).reshape(B, Sq, D),
        dxkv=(dk2 @ wk.T + dv2 @ wv.T).reshape(B, L, D),
        dwq=xq2.T @ dq2, dwk=xkv2.T @ dk2, dwv=xkv2.T @ dv2, dwo=dwo,
        dq=dq, dk=dk, dv=dv, do=do, delta=delta,
        y=fw["y"], lse=fw["lse"], o=o, q=q, k=k, v=v)



# --------------------------------------------------------------------------
# One window offset per batch entry (section 4.2: the windows start "at a
# random minor offset"; the paper does not say whether the offset is drawn per
# step or per sequence -- with one value per sequence every batch entry simply
# has its own early-stage mask).  Written as that sentence: sample by sample.
# --------------------------------------------------------------------------
def xattn_forward_sample_eps(xq, xkv, wq, wk, wv, wo, *, n_q_heads, n_kv_heads, k, eps_list, scale=None, rope=None):
    """xattn_forward with batch entry b under dense_mask(Sq, L, k, eps_list[b])."""
    xq, xkv = np.asarray(xq, F64), np.asarray(xkv, F64)
    if len(eps_list) != xq.shape[0]:
        raise ValueError("one offset per batch entry")
    parts = [xattn_forward(xq[b:b + 1], xkv[b:b + 1], wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                           mask=dense_mask(xq.shape[1], xkv.shape[1], k, int(eps_list[b])), scale=scale, rope=rope)
             for b in range(xq.shape[0])]
    out = {n: np.concatenate([p[n] for p in parts], axis=0) for n in ("y", "lse", "q", "k", "v", "o")}
    out["scale"] = parts[0]["scale"]
    return out


def xattn_backward_sample_eps(dy, xq, xkv, wq, wk, wv, wo, *, n_q_heads, n_kv_heads, k, eps_list, scale=None,
                              rope=None):
    """Gradients under per-entry offsets: input gradients entry by entry, weight
    gradients summed over the entries (the loss is a sum over the batch)."""
    dy, xq, xkv = np.asarray(dy, F64), np.asarray(xq, F64), np.asarray(xkv, F64)
    if len(eps_list) != xq.shape[0]:
        raise ValueError("one offset per batch entry")
    parts = [xattn_backward(dy[b:b + 1], xq[b:b + 1], xkv[b:b + 1], wq, wk, wv, wo, n_q_heads=n_q_heads,
                            n_kv_heads=n_kv_heads, mask=dense_mask(xq.shape[1], xkv.shape[1], k, int(eps_list[b])),
                            scale=scale, rope=rope) for b in range(xq.shape[0])]
    out = {n: np.concatenate([p[n] for p in parts], axis=0) for n in ("dxq", "dxkv", "y", "lse", "o", "q", "k", "v")}
    for n in ("dwq", "dwk", "dwv", "dwo"):
        out[n] = sum(p[n] for p in parts)
    return out


# --------------------------------------------------------------------------
# Packed batches of sequences of different lengths (no padding rows): the
# training inputs are conversations of unequal length.  xq is [Tq, D] with
# sequence b in rows cu_q[b] .. cu_q[b+1]-1, xkv likewise with cu_kv.  Every
# sequence is an independent instance of Eq. 2 under its own early-stage mask;
# the weights are shared, so their gradients add up.  Written as that sentence.
# --------------------------------------------------------------------------
def _check_cu(cu, total):
    cu = [int(v) for v in cu]
    if len(cu) < 2 or cu[0] != 0 or cu[-1] != total or any(b <= a for a, b in zip(cu, cu[1:])):
        raise ValueError("cu_seqlens must start at 0, end at the row count and increase (no empty sequence)")
    return cu


def xattn_forward_packed(xq, xkv, wq, wk, wv, wo, cu_q, cu_kv, *, n_q_heads, n_kv_heads, k, eps_list=None, scale=None,
                         rope=None):
    """Returns y [Tq, D], lse [H, Tq], q [Tq, H, d], k, v [Tkv, G, d], o [Tq, H, d].  eps_list: one offset per
    sequence (default 0).  rope: positions restart at 0 in every sequence."""
    xq, xkv = np.asarray(xq, F64), np.asarray(xkv, F64)
    cu_q, cu_kv = _check_cu(cu_q, xq.shape[0]), _check_cu(cu_kv, xkv.shape[0])
    if len(cu_q) != len(cu_kv):
        raise ValueError("as many query sequences as key sequences")
    B = len(cu_q) - 1
    parts = []
    for b in range(B):
        a, e = xq[None, cu_q[b]:cu_q[b + 1]], xkv[None, cu_kv[b]:cu_kv[b + 1]]
        eps = 0 if eps_list is None else int(eps_list[b])
        parts.append(xattn_forward(a, e, wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                                   mask=dense_mask(a.shape[1], e.shape[1], k, eps), scale=scale, rope=rope))
    out = {n: np.concatenate([p[n][0] for p in parts], axis=0) for n in ("y", "q", "k", "v", "o")}
    out["lse"] = np.concatenate([p["lse"][0] for p in parts], axis=1)
    return out


def xattn_backward_packed(dy, xq, xkv, wq, wk, wv, wo, cu_q, cu_kv, *, n_q_heads, n_kv_heads, k, eps_list=None,
                          scale=None, rope=None):
    """Gradients for packed sequences: dxq [Tq, D], dxkv [Tkv, D], weight gradients summed over the sequences."""
    dy, xq, xkv = np.asarray(dy, F64), np.asarray(xq, F64), np.asarray(xkv, F64)
    cu_q, cu_kv = _check_cu(cu_q, xq.shape[0]), _check_cu(cu_kv, xkv.shape[0])
    B = len(cu_q) - 1
    parts = []
    for b in range(B):
        sq, sk = slice(cu_q[b], cu_q[b + 1]), slice(cu_kv[b], cu_kv[b + 1])
        eps = 0 if eps_list is None else int(eps_list[b])
        parts.append(xattn_backward(dy[None, sq], xq[None, sq], xkv[None, sk], wq, wk, wv, wo, n_q_heads=n_q_heads,
                                    n_kv_heads=n_kv_heads, mask=dense_mask(sq.stop - sq.start, sk.stop - sk.start, k, eps),
                                    scale=scale, rope=rope))
    out = {n: np.concatenate([p[n][0] for p in parts], axis=0) for n in ("dxq", "dxkv", "y", "o", "q", "k", "v")}
    out["lse"] = np.concatenate([p["lse"][0] for p in parts], axis=1)
    for n in ("dwq", "dwk", "dwv", "dwo"):
        out[n] = sum(p[n] for p in parts)
    return out

# --------------------------------------------------------------------------
# Late-stage training: simulated inference steps (section 4.2, second half, and
# the caption of the mask figure; the figure itself is not available)
#
# The keys of a query come from two sources: the true target states Xkv, under
# the early-stage mask, and a buffer Xp of states that the draft model itself
# predicted in the earlier simulation steps of this training iteration (one
# buffer of the sequence's size, updated in place: "constant space").  After t
# steps the first t positions of every window hold predicted states, and a
# query may use those of its own window that lie before it.
#
# Readings taken here (PARITY UNPINNED by the paper beyond the prose: the
# figure that defines the masks is missing from the text):
#   * step t >= 0; t = 0 is the early-stage mask (no predicted key visible);
#   * query p, whose window starts at w0(p) = eps + k*floor((p - eps)/k) (below
#     zero for the partial leading window), sees predicted key j iff
#     max(w0(p), 0) <= j < min(p, w0(p) + t): positions are counted from the
#     window's own start also in the leading partial window;
#   * queries are not unrolled: Xq is the same in every step;
#   * K and V of the predicted states use the same Wk, Wv as the true states.
# --------------------------------------------------------------------------
def sim_pred_mask_loops(seq_q: int, seq_kv: int, k: int, eps: int, t: int) -> np.ndarray:
    """Boolean [seq_q, seq_kv]: True where query p may attend PREDICTED key j at
    simulation step t.  Element by element from the prose: inside each window,
    the states predicted so far are those of its first t positions, and a query
    reaches the ones strictly before itself."""
    if t < 0:
        raise ValueError("simulation step must be >= 0")
    m = np.zeros((seq_q, seq_kv), dtype=bool)
    for n in _window_starts(seq_q, k, eps):
        for p in range(max(n, 0), min(n + k, seq_q)):
            for j in range(max(n, 0), min(n + k, seq_kv)):
                if j < p and j - n < t:
                    m[p, j] = True
    return m


def sim_pred_mask(seq_q: int, seq_kv: int, k: int, eps: int, t: int) -> np.ndarray:
    """Same mask as sim_pred_mask_loops from the closed form
    max(w0(p), 0) <= j < min(p, w0(p) + t), affordable at full size."""
    if t < 0 or k < 1 or not (0 <= eps < k):
        raise ValueError("need t >= 0, k >= 1 and 0 <= eps < k")
    p = np.arange(seq_q)[:, None]
    j = np.arange(seq_kv)[None, :]
    w0 = eps + k * np.floor_divide(p - eps, k)
    return (j >= np.maximum(w0, 0)) & (j < np.minimum(p, w0 + t))



def sim_save_predicted(xpred, h, k: int, eps: int, t: int) -> np.ndarray:
    """In-place update between simulation steps (section 4.2, second half: the
    states predicted at the start of every window are saved after the first
    step, those of the next position after the second step, and so on, into
    the one buffer).  After step t (t = 0 is the early-stage step) the rows
    whose position inside their window is t take the newly predicted states h
    of the same positions; every other row of the buffer keeps its content.
    Returns the updated copy of xpred.  Window by window, row by row, as in
    the prose; the leading partial window counts positions from its own
    (negative) start, as sim_pred_mask_loops does.  PARITY UNPINNED by the
    paper beyond the prose (the figure is missing)."""
    xpred, h = np.array(xpred, F64, copy=True), np.asarray(h, F64)
    if xpred.shape != h.shape:
        raise ValueError("h and the predicted-state buffer must have the same shape")
    if t < 0 or k < 1 or not (0 <= eps < k):
        raise ValueError("need t >= 0, k >= 1 and 0 <= eps < k")
    L = xpred.shape[1]
    for n in _window_starts(L, k, eps):
        j = n + t
        if t < k and 0 <= j < L:
            xpred[:, j] = h[:, j]
    return xpred

def _sim_concat(xkv, xpred, k, eps, t, seq_q):
    xkv, xpred = np.asarray(xkv, F64), np.asarray(xpred, F64)
    if xkv.shape != xpred.shape:
        raise ValueError("the predicted-state buffer has the shape of the target states")
    L = xkv.shape[1]
    mask = np.concatenate([dense_mask(seq_q, L, k, eps), sim_pred_mask(seq_q, L, k, eps, t)], axis=1)
    return np.concatenate([xkv, xpred], axis=1), mask, L


def _sim_rope(rope, L):
    """A predicted state stands at its own sequence position: the concatenated keys have positions 0..L-1 twice."""
    if rope is None:
        return None
    return dict(base=rope.get("base"), q_pos=None, k_pos=np.concatenate([np.arange(L), np.arange(L)]))


def xattn_forward_sim(xq, xkv, xpred, wq, wk, wv, wo, *, n_q_heads, n_kv_heads, k, eps, t, scale=None, rope=None):
    """Forward of simulation step t: Eq. 2 over the keys [true states under the
    early-stage mask | predicted states under sim_pred_mask].  Returns the dict
    of xattn_forward with k, v split into k, v (true) and kp, vp (predicted)."""
    cat, mask, L = _sim_concat(xkv, xpred, k, eps, t, np.asarray(xq).shape[1])
    out = xattn_forward(xq, cat, wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, mask=mask, scale=scale,
                        rope=_sim_rope(rope, L))
    out["kp"], out["vp"] = out["k"][:, L:], out["v"][:, L:]
    out["k"], out["v"] = out["k"][:, :L], out["v"][:, :L]
    return out


def xattn_backward_sim(dy, xq, xkv, xpred, wq, wk, wv, wo, *, n_q_heads, n_kv_heads, k, eps, t, scale=None,
                       rope=None):
    """Gradients of simulation step t with respect to every input, the
    predicted-state buffer included (dxpred; zero on rows that no query sees)."""
    cat, mask, L = _sim_concat(xkv, xpred, k, eps, t, np.asarray(xq).shape[1])
    out = xattn_backward(dy, xq, cat, wq, wk, wv, wo, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, mask=mask,
                         scale=scale, rope=_sim_rope(rope, L))
    out["dxpred"] = out["dxkv"][:, L:]
    out["dxkv"] = out["dxkv"][:, :L]
    for n in ("k", "v", "dk", "dv"):
        out[n + "p"], out[n] = out[n][:, L:], out[n][:, :L]
    return out


# --------------------------------------------------------------------------
# Decode-time draft step (section 4.1, KV-cache paragraph)
# --------------------------------------------------------------------------
def draft_step(x, k_cache, v_cache, wq, wo, *, n_q_heads, n_kv_heads, scale=None, rope=None):
    """M draft queries against a cache of L already-projected K/V rows.

    x [M, D]; k_cache, v_cache [L, G, d]; every query sees every cache row
    (drafted states are not concatenated).  rope: None or dict(base, q_pos [M]):
    the projected queries are rotated to those positions (the cache rows were
    rotated when they were appended).  Returns y [M, D], lse [H, M].
    """
    x = np.asarray(x, F64)
    kc, vc = np.asarray(k_cache, F64), np.asarray(v_cache, F64)
    wq, wo = np.asarray(wq, F64), np.asarray(wo, F64)
    H, G = n_q_heads, n_kv_heads
    rep = _check_heads(H, G)
    M, D = x.shape
    L, _, d = kc.shape
    if scale is None or scale == 0:
        scale = 1.0 / math.sqrt(d)
    q = (x @ wq).reshape(M, H, d)
    if rope is not None:
        q = rope_rotate(q, rope["q_pos"], rope.get("base", 10000.0) or 10000.0)
    o = np.zeros((M, H, d), F64)
    lse = np.zeros((H, M), F64)
    allvis = np.ones((M, L), bool)
    for h in range(H):
        g = h // rep
        s = (q[:, h, :] @ kc[:, g, :].T) * scale
        P, lse[h] = masked_softmax(s, allvis)
        o[:, h, :] = P @ vc[:, g, :]
    y = o.reshape(M, H * d) @ wo
    return dict(y=y, lse=lse, q=q, o=o)


# --------------------------------------------------------------------------
# Decode with drafted states concatenated to the cache, under a draft tree
# (section 4.1, KV-cache paragraph: newly drafted states' K and V rows are
# appended as drafting proceeds and the cache goes back to the true states
# when a speculative-decoding iteration ends; appendix "Ablation Study": the
# "concate" option and the dynamic drafting tree; section 5.1: its shape,
# depth 1+6, top-k 10, 60 candidates)
#
# Readings taken here (the paper gives no formula for the tree mask):
#   * The cache holds n_true rows of true target states followed by the rows
#     of the states drafted so far in this iteration, in the order they were
#     appended.  Every query sees every true row.
#   * A query placed at draft node t sees the drafted rows of the PROPER
#     ancestors of t only: its own state is appended after the query has run
#     (the section 4.1 wording), and siblings / other branches never.
#     PARITY UNPINNED by the paper beyond that wording; the entry point takes
#     an arbitrary boolean mask, ancestor_mask() builds this reading of it.
#   * Resetting the cache is dropping the rows past n_true: no arithmetic.
# --------------------------------------------------------------------------
def kv_project(x_new, wk, wv, *, n_kv_heads, rope=None):
    """K and V rows of n new states (true or drafted): x_new [n, D] -> [n, G, d] each.
    rope: None or dict(base, k_pos [n]) -- the sequence positions of the new states, to which K is rotated."""
    x = np.asarray(x_new, F64)
    wk, wv = np.asarray(wk, F64), np.asarray(wv, F64)
    n = x.shape[0]
    G = n_kv_heads
    if wk.shape[1] % G or wk.shape != wv.shape:
        raise ValueError("K/V weight shapes")
    d = wk.shape[1] // G
    kn = (x @ wk).reshape(n, G, d)
    if rope is not None:
        kn = rope_rotate(kn, rope["k_pos"], rope.get("base", 10000.0) or 10000.0)
    return kn, (x @ wv).reshape(n, G, d)


def kv_append(k_cache, v_cache, pos, x_new, wk, wv, *, n_kv_heads, rope=None):
    """Copies of the caches with rows pos .. pos+n-1 replaced by the K/V rows of x_new."""
    kc, vc = np.array(k_cache, F64, copy=True), np.array(v_cache, F64, copy=True)
    kn, vn = kv_project(x_new, wk, wv, n_kv_heads=n_kv_heads, rope=rope)
    n = kn.shape[0]
    if pos < 0 or pos + n > kc.shape[0]:
        raise ValueError("append range outside the cache")
    kc[pos:pos + n] = kn
    vc[pos:pos + n] = vn
    return kc, vc


def ancestor_mask(parents, query_nodes):
    """Tree mask of the reading above.

    parents[t] is the parent draft node of draft node t (appended earlier, so
    parents[t] < t), or -1 when its parent is the last true token.  Returns a
    boolean [len(query_nodes), len(parents)] matrix: entry (m, t) is True iff
    node t is a proper ancestor of node query_nodes[m].
    """
    T = len(parents)
    for t, p in enumerate(parents):
        if not (-1 <= p < t):
            raise ValueError("parents must point to earlier nodes or -1")
    out = np.zeros((len(query_nodes), T), bool)
    for m, node in enumerate(query_nodes):
        if not (0 <= node < T):
            raise ValueError("query node out of range")
        a = parents[node]
        while a >= 0:
            out[m, a] = True
            a = parents[a]
    return out


def draft_step_tree(x, k_cache, v_cache, wq, wo, *, n_true, tree_mask, n_q_heads, n_kv_heads, scale=None, rope=None):
    """M draft queries against n_true true rows plus T drafted rows of the cache.

    x [M, D]; k_cache, v_cache [n_true + T, G, d]; tree_mask boolean [M, T]:
    query m sees every true row, and drafted row n_true + t iff tree_mask[m, t].
    Returns y [M, D], lse [H, M].
    """
    x = np.asarray(x, F64)
    kc, vc = np.asarray(k_cache, F64), np.asarray(v_cache, F64)
    wq, wo = np.asarray(wq, F64), np.asarray(wo, F64)
    tm = np.asarray(tree_mask, bool)
    H, G = n_q_heads, n_kv_heads
    rep = _check_heads(H, G)
    M, D = x.shape
    L, _, d = kc.shape
    T = L - n_true
    if n_true < 0 or T < 0 or tm.shape != (M, T):
        raise ValueError("tree mask must be [M, rows past n_true]")
    if scale is None or scale == 0:
        scale = 1.0 / math.sqrt(d)
    vis = np.concatenate([np.ones((M, n_true), bool), tm], axis=1)
    q = (x @ wq).reshape(M, H, d)
    if rope is not None:
        q = rope_rotate(q, rope["q_pos"], rope.get("base", 10000.0) or 10000.0)
    o = np.zeros((M, H, d), F64)
    lse = np.zeros((H, M), F64)
    for h in range(H):
        g = h // rep
        s = (q[:, h, :] @ kc[:, g, :].T) * scale
        P, lse[h] = masked_softmax(s, vis)
        o[:, h, :] = P @ vc[:, g, :]
    y = o.reshape(M, H * d) @ wo
    return dict(y=y, lse=lse, q=q, o=o)


# --------------------------------------------------------------------------
# Accounting helpers used by the tests and the benchmark's CPU leg
# --------------------------------------------------------------------------
def visible_pairs(mask: np.ndarray) -> int:
    return int(np.asarray(mask, bool).sum())
