"""GPU parity of the draft step on prepared (packed) projection weights against the float64 oracle
(section 4.1, KV-cache paragraph; appendix "Ablation Study" for the tree variant): the same definition of y and LSE
as the plain draft step, so the same oracle functions and the same tolerances; plus the packing itself (exact,
against the layout the header documents),
agreement with the plain entry point, and the shapes the prepared path refuses."""
import numpy as np
import pytest

from oracle import beagle_oracle as orc
from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth
from gpu_harness import run_draft_prepared, run_draft_tree, packed_strips, max_abs, rel_fro
from test_gpu_tree_decode import _problem, _random_tree, BF16_OUT_ABS, BF16_OUT_FRO, LSE_TOL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,n_true,T,H,G,D", [
    (1, 1000, 0, 4, 4, 512),          # one query: the merge of the key ranges rides in the projection
    (1, 130, 40, 4, 2, 512),
    (1, 4096, 0, 32, 32, 4096),       # the decode configuration
    (2, 900, 0, 4, 4, 512), (4, 1000, 17, 8, 8, 1024), (5, 640, 0, 4, 1, 512),
    (8, 1000, 31, 4, 2, 512), (9, 1000, 0, 4, 4, 512), (10, 4096, 50, 32, 32, 4096), (16, 777, 33, 8, 8, 1024),
    (8, 300, 0, 36, 36, 4608),        # K past 4096 in the 8-row layout; waves with four and with five macro-steps
    (5, 300, 0, 72, 72, 512),         # nine macro-steps per wave: activations parked chunk by chunk, three rounds
    (12, 300, 0, 40, 40, 640),        # the same in the 16-row layout (K = 5120: five macro-steps per wave)
    (9, 200, 0, 33, 33, 512),         # 33 heads: one wave has five macro-steps, the others four
    (3, 500, 0, 9, 9, 1152),          # waves with one and with two macro-steps
    (11, 500, 20, 5, 5, 640),         # K = 640: three waves without any
    (7, 0, 90, 4, 4, 512),            # no true row at all
])
def test_prepared_step_matches_the_oracle(M, n_true, T, H, G, D):
    rng = np.random.default_rng(300 + M + T)
    cfg, inp, kc, vc = _problem("bf16", M, n_true + T, H, G, D, 128, 1800 + M)
    if T:
        parents = _random_tree(rng, T)
        tm = orc.ancestor_mask(parents, [int(v) for v in rng.integers(0, T, M)])
        if M > 1:
            tm[M // 2] = rng.random(T) < 0.5
    else:
        tm = np.zeros((M, 0), bool)
    ref = orc.draft_step_tree(inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true=n_true, tree_mask=tm,
                              n_q_heads=H, n_kv_heads=G)
    y, lse, (wq_pk, wo_pk) = run_draft_prepared(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true, tm)
    assert np.array_equal(wq_pk, packed_strips(inp["wq"]))      # packing moves values, nothing else
    assert np.array_equal(wo_pk, packed_strips(inp["wo"]))
    fin = np.isfinite(ref["lse"])
    assert np.array_equal(np.isneginf(lse), ~fin)
    assert np.isfinite(y).all()
    assert max_abs(y, ref["y"]) <= BF16_OUT_ABS and rel_fro(y, ref["y"]) <= BF16_OUT_FRO, rel_fro(y, ref["y"])
    assert max_abs(lse[fin], ref["lse"][fin]) <= LSE_TOL
    assert (y[~fin.any(axis=0)] == 0).all()
    # and next to the plain entry point: both differ by the order of the projections' sums only
    y0, l0 = run_draft_tree(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], n_true, tm)
    assert max_abs(l0[fin], lse[fin]) <= 1e-4
    assert max_abs(y, y0) <= 2.0 ** -7 * max(1.0, float(np.abs(y0).max()))


@pytest.mark.parametrize("M,H,D,dtype", [(17, 4, 512, "bf16"), (64, 4, 512, "bf16"), 
                                         (4, 4, 520, "bf16"), (3, 4, 256, "f32")])
def test_shapes_outside_the_prepared_path_are_refused(M, H, D, dtype):
    d = 128 if dtype == "bf16" else 64
    cfg, inp, kc, vc = _problem(dtype, M, 64, H, H, D, d, 1900)
    st = run_draft_prepared(cfg, inp["xq"][0], kc, vc, inp["wq"], inp["wo"], 64, np.zeros((M, 0), bool), check=False)
    assert st == bx.BEAGLE_ERR_UNSUPPORTED


def test_prepared_step_in_a_hip_graph_replays_to_the_eager_result():
    import torch
    import gpu_harness as gh
    M, L, H, D = 10, 1500, 8, 1024
    cfg = synth.CONFIGS["c4"].with_(seq_q=M, seq_kv=L, hidden=D, n_q_heads=H, n_kv_heads=H)
    desc = gh.desc_of(cfg)
    g = torch.Generator(device=gh.DEV).manual_seed(77)
    R = lambda *s, std=1.0: (torch.randn(*s, device=gh.DEV, generator=g) * std).to(torch.bfloat16)
    x, kc, vc, wq, wo = R(M, D), R(L, H, 128, std=1.28), R(L, H, 128, std=1.28), R(D, H * 128, std=0.02), R(H * 128, D, std=0.02)
    wq_pk = torch.empty(D * H * 128, dtype=torch.bfloat16, device=gh.DEV)
    wo_pk = torch.empty(D * H * 128, dtype=torch.bfloat16, device=gh.DEV)
    bx.beagle_xattn_prepare_weights(desc, wq=wq, wo=wo, wq_pk=wq_pk, wo_pk=wo_pk)
    ws, ws_g = gh.workspace(desc, bx.BEAGLE_WS_DRAFT), gh.workspace(desc, bx.BEAGLE_WS_DRAFT)
    y_e = torch.full((M, D), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    l_e = torch.full((H, M), float("nan"), dtype=torch.float32, device=gh.DEV)
    bx.beagle_xattn_draft_step_prepared(desc, x, kc, vc, wq_pk, wo_pk, L, None, 0, y_e, l_e, ws)
    torch.cuda.synchronize()
    y_g, l_g = torch.empty_like(y_e), torch.empty_like(l_e)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        bx.beagle_xattn_draft_step_prepared(desc, x, kc, vc, wq_pk, wo_pk, L, None, 0, y_g, l_g, ws_g, torch.cuda.current_stream())
    for rep in range(3):
        y_g.fill_(float("nan")); l_g.fill_(float("nan"))
        gr.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g.view(torch.int16), y_e.view(torch.int16)) and torch.equal(l_g, l_e), rep
        bx.beagle_xattn_draft_step_prepared(desc, x, kc, vc, wq_pk, wo_pk, L, None, 0, y_e, l_e, ws)   # eager work in between
        torch.cuda.synchronize()


@pytest.mark.parametrize("n,pos,cap,G,D", [(1, 4096, 4200, 32, 4096), (10, 37, 300, 4, 512), (16, 100, 160, 2, 1024),
                                           (7, 11, 64, 2, 896), (9, 0, 9, 1, 640)])
def test_kv_append_on_packed_weights(n, pos, cap, G, D):
    """beagle_xattn_kv_append_prepared against the oracle's kv_append; rows outside [pos, pos + n) stay as they were."""
    import torch
    import gpu_harness as gh
    d = 128
    rng = np.random.default_rng(n + pos)
    cfg, inp, _, _ = _problem("bf16", n, cap, G, G, D, d, 1900 + n)
    x_new = inp["xq"][0]
    old_k = synth.round_to_bf16(rng.standard_normal((cap, G, d)).astype(np.float32))
    old_v = synth.round_to_bf16(rng.standard_normal((cap, G, d)).astype(np.float32))
    wantk, wantv = orc.kv_append(old_k, old_v, pos, x_new, inp["wk"], inp["wv"], n_kv_heads=G)
    desc = gh.desc_of(cfg)
    t = {k: gh.to_dev(a, cfg) for k, a in dict(x=x_new, wk=inp["wk"], wv=inp["wv"], kc=old_k, vc=old_v).items()}
    wk_pk = torch.full((D * G * d,), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    wv_pk = torch.full((D * G * d,), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    bx.beagle_xattn_prepare_weights(desc, wk=t["wk"], wv=t["wv"], wk_pk=wk_pk, wv_pk=wv_pk)
    assert np.array_equal(gh.to_host(wk_pk), packed_strips(inp["wk"])) and np.array_equal(gh.to_host(wv_pk), packed_strips(inp["wv"]))
    bx.beagle_xattn_kv_append_prepared(desc, t["x"], wk_pk, wv_pk, t["kc"], t["vc"], pos)
    torch.cuda.synchronize()
    gotk, gotv = gh.to_host(t["kc"]), gh.to_host(t["vc"])
    keep = np.ones(cap, bool)
    keep[pos:pos + n] = False
    assert np.array_equal(gotk[keep], old_k[keep]) and np.array_equal(gotv[keep], old_v[keep])
    for got, want in ((gotk, wantk), (gotv, wantv)):
        assert max_abs(got[pos:pos + n], want[pos:pos + n]) <= BF16_OUT_ABS
        assert rel_fro(got[pos:pos + n], want[pos:pos + n]) <= BF16_OUT_FRO


def test_kv_append_on_packed_weights_refuses_what_it_does_not_serve():
    import torch
    import gpu_harness as gh
    cfg, inp, _, _ = _problem("bf16", 17, 64, 4, 4, 512, 128, 1950)
    a = torch.zeros(1 << 20, dtype=torch.bfloat16, device=gh.DEV)
    assert bx.beagle_xattn_kv_append_prepared(gh.desc_of(cfg), a, a, a, a, a, 0, check=False) == bx.BEAGLE_ERR_UNSUPPORTED   # 17 states
    cfg2 = cfg.with_(seq_q=4)
    assert bx.beagle_xattn_kv_append_prepared(gh.desc_of(cfg2), a, a, a, a, a, 61, check=False) == bx.BEAGLE_ERR_SHAPE        # past the end
    assert bx.beagle_xattn_kv_append_prepared(gh.desc_of(cfg2), a, None, a, a, a, 0, check=False) == bx.BEAGLE_ERR_NULL
