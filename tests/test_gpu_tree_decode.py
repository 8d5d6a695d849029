"""GPU parity of the decode extensions -- drafted states concatenated to the
cache under a draft-tree mask, and appending states to the cache -- against
the float64 oracle (section 4.1 KV-cache paragraph; appendix "Ablation Study", "concate" with
the dynamic drafting tree).  Inputs are seeded and synthetic; trees have the
shape the paper states for its evaluation (depth 1 + 6, top-k 10, at most 60
drafted nodes) or are random."""
import numpy as np
import pytest
import torch

from oracle import beagle_oracle as orc
from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth
from gpu_harness import run_draft_tree, run_kv_append, run_draft, max_abs, rel_fro, rel_max

pytestmark = pytest.mark.gpu

F32_TOL = 1e-5
BF16_OUT_ABS, BF16_OUT_FRO, LSE_TOL = 2e-2, 1e-2, 1e-3


def _random_tree(rng, T):
    return [int(rng.integers(-1, t)) for t in range(T)]


def _problem(dtype, M, rows, H, G, D, d, seed):
    """Inputs of the decode recipe (c4): normalised states, N(0, 0.02^2) weights; the cache rows are the
    oracle's projection of the states, stored in the io dtype."""
    base = synth.CONFIGS["c4" if dtype == "bf16" else "c1"]
    cfg = base.with_(batch=1, seq_q=M, seq_kv=rows, hidden=D, n_q_heads=H, n_kv_heads=G, head_dim=d, seed_base=seed)
    inp = synth.make_inputs(cfg, with_dy=False)
    xkv = inp["xkv"][0].astype(np.float64)
    kc = (xkv @ inp["wk"]).astype(np.float32).reshape(rows, G, d)
    vc = (xkv @ inp["wv"]).astype(np.float32).reshape(rows, G, d)
    if dtype == "bf16":
        kc, vc = synth.round_to_bf16(kc), synth.round_to_bf16(vc)
    return cfg, inp, kc, vc


# ------------------------------------------------------------------ fp32
@pytest.mark.parametrize("M,n_true,T,H,G", [(6, 40, 9, 4, 2), (3, 0, 5, 4, 4), (5, 70, 0, 4, 4), (9, 33, 64, 2, 1)])
def test_fp32_tree_step(M, n_true, T, H, G):
    rng = np.random.default_rng(100 + M)
    cfg, inp, kc, vc = _problem("f32", M, n_true + T, H, G, 256, 64, 700 + M)
    tm = rng.random((M, T)) < 0.4
    if T:
        tm[0] = False                                          # one query sees no drafted row at all
    ref = orc.draft_step_tree(inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true=n_true, tree_mask=tm,
                              n_q_heads=H, n_kv_heads=G)
    y, lse = run_draft_tree(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true, tm)
    assert rel_max(y, ref["y"]) <= F32_TOL
    fin = np.isfinite(ref["lse"])
    assert np.array_equal(np.isneginf(lse), ~fin)
    assert max_abs(lse[fin], ref["lse"][fin]) <= F32_TOL * max(1.0, np.abs(ref["lse"][fin]).max()) if fin.any() else True
    if n_true == 0 and T:
        assert (y[0] == 0).all() and np.isneginf(lse[:, 0]).all()   # sees nothing: zero row, LSE -inf


# ------------------------------------------------------------------ bf16, reduced sizes
@pytest.mark.parametrize("M,n_true,T,H,G,D", [
    (1, 1000, 1, 4, 4, 512), (7, 1000, 31, 4, 2, 512), (20, 777, 33, 8, 8, 1024), (40, 600, 60, 4, 4, 512),
    (10, 1024, 200, 4, 1, 512),      # drafted rows span several 128-key steps and two key ranges
    (4, 0, 90, 4, 4, 512),           # no true row at all
    (8, 500, 0, 4, 4, 512),          # no drafted row: the plain step
    (64, 130, 30, 4, 4, 512),
])
def test_bf16_tree_step(M, n_true, T, H, G, D):
    rng = np.random.default_rng(200 + M + T)
    cfg, inp, kc, vc = _problem("bf16", M, n_true + T, H, G, D, 128, 800 + M)
    if T:
        parents = _random_tree(rng, T)
        nodes = [int(v) for v in rng.integers(0, T, M)]
        tm = orc.ancestor_mask(parents, nodes)
        tm[M // 2] = rng.random(T) < 0.5                       # and one arbitrary row
    else:
        tm = np.zeros((M, 0), bool)
    ref = orc.draft_step_tree(inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true=n_true, tree_mask=tm,
                              n_q_heads=H, n_kv_heads=G)
    y, lse = run_draft_tree(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true, tm)
    fin = np.isfinite(ref["lse"])
    assert np.array_equal(np.isneginf(lse), ~fin)
    assert np.isfinite(y).all()
    assert max_abs(y, ref["y"]) <= BF16_OUT_ABS and rel_fro(y, ref["y"]) <= BF16_OUT_FRO, rel_fro(y, ref["y"])
    assert max_abs(lse[fin], ref["lse"][fin]) <= LSE_TOL
    blind = ~fin.any(axis=0)
    assert (y[blind] == 0).all()


def test_bf16_tree_step_full_mask_equals_plain_step_bitwise():
    M, rows = 12, 900
    cfg, inp, kc, vc = _problem("bf16", M, rows, 4, 4, 512, 128, 850)
    y0, l0 = run_draft(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"])
    y1, l1 = run_draft_tree(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], 700, np.ones((M, 200), bool))
    assert np.array_equal(y0, y1) and np.array_equal(l0, l1)


# ------------------------------------------------------------------ the paper's tree shape at the decode config
def test_c4_tree_step_paper_shaped_tree():
    """L = 4096 true rows + 50 drafted rows (depth 1 + 5 done, top-k 10 per depth), the 10 queries of the last
    depth; H32/G32, D 4096."""
    rng = np.random.default_rng(7)
    depth_nodes, parents = [], []
    for dpt in range(5):
        first = len(parents)
        for i in range(10):
            parents.append(-1 if dpt == 0 else int(rng.choice(depth_nodes[-1])))
        depth_nodes.append(list(range(first, first + 10)))
    T, M, n_true = len(parents), 10, 4096
    # the queries of the next depth hang below nodes of the last finished depth: they see that node AND its ancestors
    anchors = [int(rng.choice(depth_nodes[-1])) for _ in range(M)]
    tm = orc.ancestor_mask(parents, anchors)
    for m, a in enumerate(anchors):
        tm[m, a] = True
    cfg, inp, kc, vc = _problem("bf16", M, n_true + T, 32, 32, 4096, 128, 400)
    ref = orc.draft_step_tree(inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true=n_true, tree_mask=tm,
                              n_q_heads=32, n_kv_heads=32)
    y, lse = run_draft_tree(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true, tm)
    assert max_abs(y, ref["y"]) <= BF16_OUT_ABS and rel_fro(y, ref["y"]) <= BF16_OUT_FRO
    assert max_abs(lse, ref["lse"]) <= LSE_TOL


# ------------------------------------------------------------------ kv_append
@pytest.mark.parametrize("dtype,n,pos,cap,G,D,d", [
    ("f32", 5, 3, 20, 2, 256, 64), ("f32", 1, 0, 1, 4, 256, 64),
    ("bf16", 1, 4096, 4200, 32, 4096, 128), ("bf16", 10, 37, 300, 4, 512, 128), ("bf16", 60, 100, 160, 2, 1024, 128),
    ("bf16", 300, 0, 300, 8, 512, 128),
    ("bf16", 7, 11, 64, 2, 832, 128), ("bf16", 40, 0, 40, 1, 320, 128),   # partial last k-slice; two blocks of states
])
def test_kv_append(dtype, n, pos, cap, G, D, d):
    rng = np.random.default_rng(n + pos)
    H = G
    cfg, inp, _, _ = _problem(dtype, n, cap, H, G, D, d, 900 + n)
    x_new = inp["xq"][0]                                        # n states of the recipe (stored values)
    old_k = rng.standard_normal((cap, G, d)).astype(np.float32)
    old_v = rng.standard_normal((cap, G, d)).astype(np.float32)
    if dtype == "bf16":
        old_k, old_v = synth.round_to_bf16(old_k), synth.round_to_bf16(old_v)
    wantk, wantv = orc.kv_append(old_k, old_v, pos, x_new, inp["wk"], inp["wv"], n_kv_heads=G)
    gotk, gotv = run_kv_append(cfg, x_new, inp["wk"], inp["wv"], old_k, old_v, pos)
    keep = np.ones(cap, bool)
    keep[pos:pos + n] = False
    assert np.array_equal(gotk[keep], old_k[keep].astype(np.float64)) and np.array_equal(gotv[keep], old_v[keep].astype(np.float64))
    for got, want in ((gotk, wantk), (gotv, wantv)):
        g, w = got[pos:pos + n], want[pos:pos + n]
        if dtype == "f32":
            assert rel_max(g, w) <= F32_TOL
        else:
            assert max_abs(g, w) <= BF16_OUT_ABS and rel_fro(g, w) <= BF16_OUT_FRO


def test_speculative_iteration_append_draft_reset():
    """One speculative-decoding iteration as section 4.1 describes it, through the ABI: the cache is filled with
    true states (kv_append), two tree depths are drafted with their states appended in between, then the cache
    is reset by going back to n_true.  Checked against the same sequence of oracle calls."""
    H = G = 4
    D, d, n_true, cap = 512, 128, 300, 400
    cfg, inp, _, _ = _problem("bf16", 8, cap, H, G, D, d, 950)
    rng = np.random.default_rng(11)
    states = synth.round_to_bf16(rng.standard_normal((cap, D)).astype(np.float32) * 0.9)
    zeros = np.zeros((cap, G, d), np.float32)
    # --- GPU
    ccfg = cfg.with_(seq_q=n_true)
    gk, gv = run_kv_append(ccfg, states[:n_true], inp["wk"], inp["wv"], zeros, zeros, 0)
    # --- oracle, on the values the GPU cache holds after each append (both sides then see the same cache)
    ok, ov = orc.kv_append(zeros, zeros, 0, states[:n_true], inp["wk"], inp["wv"], n_kv_heads=G)
    assert max_abs(gk, ok) <= BF16_OUT_ABS and max_abs(gv, ov) <= BF16_OUT_ABS
    parents = [-1, -1, -1, -1]
    x1 = inp["xq"][0][:4]
    tm1 = np.zeros((4, 0), bool)
    y1, _ = run_draft_tree(cfg.with_(seq_q=4, seq_kv=n_true), x1, gk[:n_true], gv[:n_true], inp["wq"], inp["wo"], n_true, tm1)
    r1 = orc.draft_step_tree(x1, gk[:n_true], gv[:n_true], inp["wq"], inp["wo"], n_true=n_true, tree_mask=tm1,
                             n_q_heads=H, n_kv_heads=G)
    assert max_abs(y1, r1["y"]) <= BF16_OUT_ABS and rel_fro(y1, r1["y"]) <= BF16_OUT_FRO
    # the drafted states of depth 1 (here: the step's outputs, as stored) join the cache
    drafted = synth.round_to_bf16(y1.astype(np.float32))
    gk2, gv2 = run_kv_append(cfg.with_(seq_q=4), drafted, inp["wk"], inp["wv"], gk.astype(np.float32), gv.astype(np.float32), n_true)
    assert np.array_equal(gk2[:n_true], gk[:n_true])
    # depth 2: eight queries, two below each depth-1 node
    x2 = inp["xq"][0][:8]
    tm2 = np.zeros((8, 4), bool)
    for m in range(8):
        tm2[m, m // 2] = True
    rows = n_true + 4
    y2, l2 = run_draft_tree(cfg.with_(seq_q=8, seq_kv=rows), x2, gk2[:rows], gv2[:rows], inp["wq"], inp["wo"], n_true, tm2)
    r2 = orc.draft_step_tree(x2, gk2[:rows], gv2[:rows], inp["wq"], inp["wo"], n_true=n_true, tree_mask=tm2,
                             n_q_heads=H, n_kv_heads=G)
    assert max_abs(y2, r2["y"]) <= BF16_OUT_ABS and rel_fro(y2, r2["y"]) <= BF16_OUT_FRO
    assert max_abs(l2, r2["lse"]) <= LSE_TOL
    # reset: a plain step over the first n_true rows is unaffected by the drafted rows behind them
    y3, _ = run_draft(cfg.with_(seq_q=4, seq_kv=n_true), x1, gk2[:n_true], gv2[:n_true], inp["wq"], inp["wo"])
    y4, _ = run_draft(cfg.with_(seq_q=4, seq_kv=n_true), x1, gk[:n_true], gv[:n_true], inp["wq"], inp["wo"])
    assert np.array_equal(y3, y4)


# ------------------------------------------------------------------ argument checks
def test_tree_and_append_argument_errors():
    cfg, inp, kc, vc = _problem("bf16", 4, 200, 4, 4, 512, 128, 990)
    tm = np.zeros((4, 50), bool)
    x = inp["xq"][0]
    assert run_draft_tree(cfg, x, kc, vc, inp["wq"], inp["wo"], 201, tm, check=False) == bx.BEAGLE_ERR_SHAPE
    assert run_draft_tree(cfg, x, kc, vc, inp["wq"], inp["wo"], -1, tm, check=False) == bx.BEAGLE_ERR_SHAPE
    # 100 drafted rows need 4 mask words; the packed 50-bit mask has 2
    assert run_draft_tree(cfg, x, kc, vc, inp["wq"], inp["wo"], 100, tm, check=False) == bx.BEAGLE_ERR_SHAPE
    d = bx.make_desc(batch=1, seq_q=4, seq_kv=200, hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128,
                     io_dtype=bx.BEAGLE_BF16)
    t = torch.zeros(4 * 512 * 64, dtype=torch.bfloat16, device="cuda:0")
    ws = torch.empty(bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_DRAFT), dtype=torch.uint8, device="cuda:0")
    lse = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    st = bx.beagle_xattn_draft_step_tree(d, t, t, t, t, t, 150, None, 2, t, lse, ws, check=False)
    assert st == bx.BEAGLE_ERR_NULL
    assert run_kv_append(cfg, x, inp["wk"], inp["wv"], kc, vc, 197, check=False) == bx.BEAGLE_ERR_SHAPE
    assert run_kv_append(cfg, x, inp["wk"], inp["wv"], kc, vc, -1, check=False) == bx.BEAGLE_ERR_SHAPE
