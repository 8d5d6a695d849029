"""Helpers for the GPU parity tests: move seeded inputs to the device, call the
C-ABI through the binding, bring results back as float64, and error metrics.
No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth

from paper_2505_24544_amd.devmem import DEV, desc_of, tdtype, to_dev, workspace  # noqa: F401  (re-exported)


def to_dev_f16(a: np.ndarray) -> torch.Tensor:
    """Upload as IEEE half (the values must already be half-representable)."""
    h = np.ascontiguousarray(a, np.float32).astype(np.float16)
    assert np.array_equal(h.astype(np.float32), np.asarray(a, np.float32)), "values are not half-representable"
    return torch.from_numpy(h).to(DEV).contiguous()


def _up(inp, names, cfg, f16_keys=()):
    return {n: (to_dev_f16(inp[n]) if n in f16_keys else to_dev(inp[n], cfg)) for n in names}


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def run_fwd(cfg, inp, flags=0, scale=0.0, poison=True):
    """Returns (device tensors dict, host float64 dict)."""
    dev, _ = run_fwd_device(cfg, inp, flags, scale, poison)
    host = {n: to_host(dev[n]) for n in ("y", "lse", "q", "k", "v", "o")}
    return dev, host


def run_fwd_device(cfg, inp, flags=0, scale=0.0, poison=True):
    """Forward through the C ABI; results stay on the device."""
    d = desc_of(cfg, flags, scale)
    dt = tdtype(cfg)
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    dev = {n: to_dev(inp[n], cfg) for n in ("xq", "xkv", "wq", "wk", "wv", "wo")}

    def out(*shape, dtype=dt):
        t = torch.empty(*shape, dtype=dtype, device=DEV)
        if poison:
            t.fill_(float("nan"))
        return t
    dev.update(y=out(B, S, D), lse=out(B, H, S, dtype=torch.float32), q=out(B, S, H, hd), k=out(B, L, G, hd),
               v=out(B, L, G, hd), o=out(B, S, H, hd))
    ws = workspace(d, bx.BEAGLE_WS_FWD)
    bx.beagle_xattn_fwd(d, dev["xq"], dev["xkv"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], dev["y"], dev["lse"],
                        dev["q"], dev["k"], dev["v"], dev["o"], ws)
    torch.cuda.synchronize()
    return dev, None


def run_bwd(cfg, inp, dev, flags=bx.BEAGLE_FLAG_NEED_DXKV, scale=0.0, poison=True):
    g = run_bwd_device(cfg, inp, dev, flags, scale, poison)
    return g, {n: to_host(t) for n, t in g.items() if t is not None}


def run_bwd_device(cfg, inp, dev, flags=bx.BEAGLE_FLAG_NEED_DXKV, scale=0.0, poison=True):
    d = desc_of(cfg, flags, scale)
    dt = tdtype(cfg)
    wdt = torch.float32 if (flags & bx.BEAGLE_FLAG_WGRAD_F32) else dt
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    dy = to_dev(inp["dy"], cfg)

    def out(*shape, dtype=dt):
        t = torch.empty(*shape, dtype=dtype, device=DEV)
        if poison:
            t.fill_(float("nan"))
        return t
    g = dict(dxq=out(B, S, D), dxkv=out(B, L, D) if (flags & bx.BEAGLE_FLAG_NEED_DXKV) else None,
             dwq=out(D, H * hd, dtype=wdt), dwk=out(D, G * hd, dtype=wdt), dwv=out(D, G * hd, dtype=wdt),
             dwo=out(H * hd, D, dtype=wdt))
    ws = workspace(d, bx.BEAGLE_WS_BWD)
    bx.beagle_xattn_bwd(d, dy, dev["xq"], dev["xkv"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], dev["q"], dev["k"],
                        dev["v"], dev["o"], dev["lse"], g["dxq"], g["dxkv"], g["dwq"], g["dwk"], g["dwv"], g["dwo"], ws)
    torch.cuda.synchronize()
    return g


def run_sim(cfg, inp, xpred, t, flags=bx.BEAGLE_FLAG_NEED_DXKV, scale=0.0, desc=None, f16_keys=()):
    """Forward + backward of late-stage simulation step t through the C ABI.
    Returns host float64 dicts (forward results, gradients)."""
    d = desc if desc is not None else desc_of(cfg, flags, scale)
    dt = tdtype(cfg)
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    dev = _up(inp, ("xq", "xkv", "wq", "wk", "wv", "wo", "dy"), cfg, f16_keys)
    dev["xp"] = to_dev(xpred, cfg)

    def out(*shape, dtype=dt):
        return torch.full(shape, float("nan"), dtype=dtype, device=DEV)
    f = dict(y=out(B, S, D), lse=out(B, H, S, dtype=torch.float32), q=out(B, S, H, hd), k=out(B, L, G, hd),
             v=out(B, L, G, hd), kp=out(B, L, G, hd), vp=out(B, L, G, hd), o=out(B, S, H, hd))
    bx.beagle_xattn_fwd_sim(d, dev["xq"], dev["xkv"], dev["xp"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], t,
                            f["y"], f["lse"], f["q"], f["k"], f["v"], f["kp"], f["vp"], f["o"],
                            workspace(d, bx.BEAGLE_WS_FWD))
    g = dict(dxq=out(B, S, D), dxkv=out(B, L, D) if (flags & bx.BEAGLE_FLAG_NEED_DXKV) else None,
             dxpred=out(B, L, D), dwq=out(D, H * hd), dwk=out(D, G * hd), dwv=out(D, G * hd), dwo=out(H * hd, D))
    bx.beagle_xattn_bwd_sim(d, dev["dy"], dev["xq"], dev["xkv"], dev["xp"], dev["wq"], dev["wk"], dev["wv"], dev["wo"],
                            f["q"], f["k"], f["v"], f["kp"], f["vp"], f["o"], f["lse"], t,
                            g["dxq"], g["dxkv"], g["dxpred"], g["dwq"], g["dwk"], g["dwv"], g["dwo"],
                            workspace(d, bx.BEAGLE_WS_BWD_SIM))
    torch.cuda.synchronize()
    return ({n: to_host(v) for n, v in f.items()}, {n: to_host(v) for n, v in g.items() if v is not None})


def run_sim_save(cfg, h, xpred, t, check=True):
    """xpred after beagle_xattn_sim_save(h, xpred, t); host arrays in, host float64 out."""
    d = desc_of(cfg)
    hd, xp = to_dev(h, cfg), to_dev(xpred, cfg)
    st = bx.beagle_xattn_sim_save(d, hd, xp, t, check=check)
    torch.cuda.synchronize()
    return to_host(xp) if check else st


def run_sim_loop(cfg, inp, xpred0, steps):
    """steps simulated forward steps on the device, the output y of each step saved into the buffer as the stand-in
    for the draft block's predicted states.  Returns ([y of every step], final buffer) as host float64."""
    d = desc_of(cfg)
    dt = tdtype(cfg)
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    dev = {n: to_dev(inp[n], cfg) for n in ("xq", "xkv", "wq", "wk", "wv", "wo")}
    xp = to_dev(xpred0, cfg)
    E = lambda *s, dtype=dt: torch.empty(*s, dtype=dtype, device=DEV)
    y, lse, q, o = E(B, S, D), E(B, H, S, dtype=torch.float32), E(B, S, H, hd), E(B, S, H, hd)
    k, v, kp, vp = (E(B, L, G, hd) for _ in range(4))
    ws = workspace(d, bx.BEAGLE_WS_FWD)
    ys = []
    for t in range(steps):
        bx.beagle_xattn_fwd_sim(d, dev["xq"], dev["xkv"], xp, dev["wq"], dev["wk"], dev["wv"], dev["wo"], t,
                                y, lse, q, k, v, kp, vp, o, ws)
        bx.beagle_xattn_sim_save(d, y, xp, t)
        torch.cuda.synchronize()
        ys.append(to_host(y))
    return ys, to_host(xp)


BLOCK_W = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
BLOCK_G = ("g_q", "g_kv", "g_mlp")


def run_block(cfg, bi, ffn, rms_eps, gains=True, flags=bx.BEAGLE_FLAG_NEED_DXKV, desc=None, f16_keys=()):
    """Forward + backward of the whole draft block through the C ABI.  bi: make_block_inputs' dict.
    Returns host float64 dicts (forward results incl. the saved tensors, gradients)."""
    sv, gr = run_block_device(cfg, bi, ffn, rms_eps, gains, flags, desc, f16_keys)
    return {n: to_host(v) for n, v in sv.items()}, {n: to_host(v) for n, v in gr.items()}


def run_block_device(cfg, bi, ffn, rms_eps, gains=True, flags=bx.BEAGLE_FLAG_NEED_DXKV, desc=None, f16_keys=()):
    """As run_block, results left on the device (forward dict includes h)."""
    d = desc if desc is not None else desc_of(cfg, flags)
    dt = tdtype(cfg)
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    dev = _up(bi, ("e", "hs", "dh") + BLOCK_W + (BLOCK_G if gains else ()), cfg, f16_keys)

    def out(*shape, dtype=dt):
        return torch.full(shape, float("nan"), dtype=dtype, device=DEV)
    f32 = torch.float32
    sv = dict(q=out(B, S, H, hd), k=out(B, L, G, hd), v=out(B, L, G, hd), o=out(B, S, H, hd),
              lse=out(B, H, S, dtype=f32), y=out(B, S, D), u=out(B, S, ffn), w=out(B, S, ffn), m=out(B, S, ffn))
    if gains:
        sv.update(xq_n=out(B, S, D), r_q=out(B * S, dtype=f32), xkv_n=out(B, L, D), r_kv=out(B * L, dtype=f32),
                  z=out(B, S, D), r_mlp=out(B * S, dtype=f32))
    h = out(B, S, D)
    params = bx.make_block_params(ffn, rms_eps, **{n: dev[n] for n in BLOCK_W + (BLOCK_G if gains else ())})
    saved = bx.make_block_saved(**sv)
    bx.beagle_xattn_block_fwd(d, params, dev["e"], dev["hs"], h, saved,
                              torch.empty(bx.beagle_xattn_block_workspace_bytes(d, ffn, bx.BEAGLE_WS_BLOCK_FWD),
                                          dtype=torch.uint8, device=DEV))
    gr = dict(de=out(B, S, D), dwq=out(D, H * hd), dwk=out(D, G * hd), dwv=out(D, G * hd), dwo=out(H * hd, D),
              dw_gate=out(D, ffn), dw_up=out(D, ffn), dw_down=out(ffn, D))
    if flags & bx.BEAGLE_FLAG_NEED_DXKV:
        gr["dhs"] = out(B, L, D)
    if gains:
        gr.update(dg_q=out(D, dtype=f32), dg_kv=out(D, dtype=f32), dg_mlp=out(D, dtype=f32))
    nws = bx.beagle_xattn_block_workspace_bytes(d, ffn, bx.BEAGLE_WS_BLOCK_BWD)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device=DEV)
    bx.beagle_xattn_block_bwd(d, params, dev["dh"], dev["e"], dev["hs"], saved, bx.make_block_grads(**gr), ws)
    torch.cuda.synchronize()
    sv["h"] = h
    return sv, gr


def run_train(cfg, inp, desc, f16_keys=()):
    """Training forward + backward through the C ABI under a caller-built descriptor (dXkv requested).
    f16_keys: inputs uploaded as IEEE half.  Returns host float64 dicts (forward results, gradients)."""
    dt = tdtype(cfg)
    B, S, L, D, H, G, hd = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    t = _up(inp, ("xq", "xkv", "wq", "wk", "wv", "wo", "dy"), cfg, f16_keys)
    out = lambda *s, dtype=dt: torch.full(s, float("nan"), dtype=dtype, device=DEV)
    f = dict(y=out(B, S, D), lse=out(B, H, S, dtype=torch.float32), q=out(B, S, H, hd), k=out(B, L, G, hd),
             v=out(B, L, G, hd), o=out(B, S, H, hd))
    bx.beagle_xattn_fwd(desc, t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], f["y"], f["lse"], f["q"], f["k"],
                        f["v"], f["o"], workspace(desc, bx.BEAGLE_WS_FWD))
    g = dict(dxq=out(B, S, D), dxkv=out(B, L, D), dwq=out(D, H * hd), dwk=out(D, G * hd), dwv=out(D, G * hd),
             dwo=out(H * hd, D))
    bx.beagle_xattn_bwd(desc, t["dy"], t["xq"], t["xkv"], t["wq"], t["wk"], t["wv"], t["wo"], f["q"], f["k"], f["v"],
                        f["o"], f["lse"], g["dxq"], g["dxkv"], g["dwq"], g["dwk"], g["dwv"], g["dwo"],
                        workspace(desc, bx.BEAGLE_WS_BWD))
    torch.cuda.synchronize()
    return {n: to_host(v) for n, v in f.items()}, {n: to_host(v) for n, v in g.items()}


def run_draft(cfg, x, kc, vc, wq, wo, scale=0.0, desc=None, check=True):
    """x [M,D], kc/vc [L,G,d], float32 arrays of stored values."""
    d = desc if desc is not None else desc_of(cfg, 0, scale)
    M, D, H = cfg.seq_q, cfg.hidden, cfg.n_q_heads
    t = {n: to_dev(a, cfg) for n, a in dict(x=x, kc=kc, vc=vc, wq=wq, wo=wo).items()}
    y = torch.full((M, D), float("nan"), dtype=tdtype(cfg), device=DEV)
    lse = torch.full((H, M), float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(d, bx.BEAGLE_WS_DRAFT)
    st = bx.beagle_xattn_draft_step(d, t["x"], t["kc"], t["vc"], t["wq"], t["wo"], y, lse, ws, check=check)
    torch.cuda.synchronize()
    if not check:
        return st
    return to_host(y), to_host(lse)


def pack_tree_mask(tree_bool):
    """bool [M, T] -> uint32 [M, max(1, ceil(T/32))] with bit (t % 32) of word t // 32."""
    tm = np.asarray(tree_bool, bool)
    M, T = tm.shape
    words = max(1, (T + 31) // 32)
    out = np.zeros((M, words), np.uint32)
    for t in range(T):
        out[:, t // 32] |= (tm[:, t].astype(np.uint32) << np.uint32(t % 32))
    return out


def run_draft_tree(cfg, x, kc, vc, wq, wo, n_true, tree_bool, scale=0.0, check=True):
    """Like run_draft with kc/vc holding n_true true rows then the drafted rows; tree_bool [M, T]."""
    d = desc_of(cfg, 0, scale)
    M, D, H = cfg.seq_q, cfg.hidden, cfg.n_q_heads
    t = {n: to_dev(a, cfg) for n, a in dict(x=x, kc=kc, vc=vc, wq=wq, wo=wo).items()}
    packed = pack_tree_mask(tree_bool)
    tm = torch.from_numpy(packed.view(np.int32)).to(DEV)
    y = torch.full((M, D), float("nan"), dtype=tdtype(cfg), device=DEV)
    lse = torch.full((H, M), float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(d, bx.BEAGLE_WS_DRAFT)
    st = bx.beagle_xattn_draft_step_tree(d, t["x"], t["kc"], t["vc"], t["wq"], t["wo"], n_true, tm, packed.shape[1],
                                         y, lse, ws, check=check)
    torch.cuda.synchronize()
    if not check:
        return st
    return to_host(y), to_host(lse)


def packed_strips(w):
    """The decode-time layout of a matrix W [K, N] as the header states it, built with plain index arithmetic:
    flat[((((m * N/16) + s) * 4 + j) * 64 + l) * 8 + e] = W[128 m + 32 j + 8 (l // 16) + e][16 s + l % 16]."""
    K, N = w.shape
    assert K % 128 == 0 and N % 16 == 0
    out = np.empty(K * N, w.dtype)
    for m in range(K // 128):
        for s in range(N // 16):
            blk = w[128 * m:128 * m + 128, 16 * s:16 * s + 16]          # [k, n]
            # k = 32 j + 8 g + e, lane l = 16 g + n
            piece = blk.reshape(4, 4, 8, 16).transpose(0, 1, 3, 2)       # [j, g, n, e]
            out[(m * (N // 16) + s) * 2048:(m * (N // 16) + s + 1) * 2048] = piece.reshape(-1)
    return out


def run_draft_prepared(cfg, x, kc, vc, wq, wo, n_true, tree_bool, scale=0.0, check=True, desc=None):
    """run_draft_tree through the prepared-weights entry points: wq and wo are packed by beagle_xattn_prepare_weights
    on the device, then beagle_xattn_draft_step_prepared runs on the results.  Also returns the packed matrices."""
    d = desc if desc is not None else desc_of(cfg, 0, scale)
    M, D, H = cfg.seq_q, cfg.hidden, cfg.n_q_heads
    t = {n: to_dev(a, cfg) for n, a in dict(x=x, kc=kc, vc=vc, wq=wq, wo=wo).items()}
    wq_pk = torch.full((D * H * cfg.head_dim,), float("nan"), dtype=tdtype(cfg), device=DEV)
    wo_pk = torch.full((D * H * cfg.head_dim,), float("nan"), dtype=tdtype(cfg), device=DEV)
    st = bx.beagle_xattn_prepare_weights(d, wq=t["wq"], wo=t["wo"], wq_pk=wq_pk, wo_pk=wo_pk, check=check)
    if not check and st != 0:
        return st
    packed = pack_tree_mask(tree_bool)
    tm = torch.from_numpy(packed.view(np.int32)).to(DEV) if packed.size else None
    y = torch.full((M, D), float("nan"), dtype=tdtype(cfg), device=DEV)
    lse = torch.full((H, M), float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(d, bx.BEAGLE_WS_DRAFT)
    st = bx.beagle_xattn_draft_step_prepared(d, t["x"], t["kc"], t["vc"], wq_pk, wo_pk, n_true, tm, packed.shape[1],
                                             y, lse, ws, check=check)
    torch.cuda.synchronize()
    if not check:
        return st
    return to_host(y), to_host(lse), (to_host(wq_pk), to_host(wo_pk))


def run_kv_append(cfg, x_new, wk, wv, kc, vc, pos, check=True, desc=None):
    """kc/vc: host arrays [capacity, G, d] (current cache contents).  Returns the caches after the call."""
    d = desc if desc is not None else desc_of(cfg, 0, 0.0)
    t = {n: to_dev(a, cfg) for n, a in dict(x=x_new, wk=wk, wv=wv, kc=kc, vc=vc).items()}
    ws = workspace(d, bx.BEAGLE_WS_APPEND)
    st = bx.beagle_xattn_kv_append(d, t["x"], t["wk"], t["wv"], t["kc"], t["vc"], pos, ws, check=check)
    torch.cuda.synchronize()
    if not check:
        return st
    return to_host(t["kc"]), to_host(t["vc"])


# ------------------------------------------------------------------ metrics
def max_abs(a, b):
    return float(np.max(np.abs(a - b))) if a.size else 0.0


def rel_max(a, ref):
    """max |a - ref| / max |ref|."""
    den = float(np.max(np.abs(ref))) if ref.size else 0.0
    return max_abs(a, ref) / den if den > 0 else max_abs(a, ref)


def rel_fro(a, ref):
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((a - ref).ravel()))
    return num / den if den > 0 else num


def lse_err(got, ref):
    """Max abs error over finite entries; the -inf pattern must agree exactly."""
    fin = np.isfinite(ref)
    assert np.array_equal(np.isneginf(got), ~fin), "empty-row pattern differs"
    return max_abs(got[fin], ref[fin]) if fin.any() else 0.0
