"""HIP-graph capture of the entry points: the library enqueues kernel launches only (no synchronisation, no
allocation, no memset), so a captured call must replay to bitwise the eager result -- also when replayed several
times with eager work of the same library in between."""
import numpy as np
import pytest
import torch

from paper_2505_24544_amd import binding as bx
from paper_2505_24544_amd import synth
import gpu_harness as gh

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _decode_tensors(M, L, H, G, D, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    bf = torch.bfloat16
    R = lambda *s, std=1.0: (torch.randn(*s, device=DEV, generator=g) * std).to(bf)
    x = R(M, D)
    return x, R(L, G, 128, std=1.28), R(L, G, 128, std=1.28), R(D, H * 128, std=0.02), R(H * 128, D, std=0.02)


@pytest.mark.parametrize("M,L,H,G,D", [(1, 4096, 32, 32, 4096), (8, 1000, 4, 2, 512), (40, 600, 4, 4, 512),
                                       (64, 4096, 32, 32, 4096)])
def test_draft_step_graph_replay_is_bitwise_the_eager_call(M, L, H, G, D):
    cfg = synth.CONFIGS["c4"].with_(seq_q=M, seq_kv=L, hidden=D, n_q_heads=H, n_kv_heads=G)
    desc = gh.desc_of(cfg)
    x, kc, vc, wq, wo = _decode_tensors(M, L, H, G, D, 31 + M)
    ws = gh.workspace(desc, bx.BEAGLE_WS_DRAFT)
    y_e = torch.full((M, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse_e = torch.full((H, M), float("nan"), dtype=torch.float32, device=DEV)
    bx.beagle_xattn_draft_step(desc, x, kc, vc, wq, wo, y_e, lse_e, ws)
    torch.cuda.synchronize()
    y_g, lse_g = torch.empty_like(y_e), torch.empty_like(lse_e)
    ws_g = gh.workspace(desc, bx.BEAGLE_WS_DRAFT)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        bx.beagle_xattn_draft_step(desc, x, kc, vc, wq, wo, y_g, lse_g, ws_g, torch.cuda.current_stream())
    for rep in range(4):
        y_g.fill_(float("nan")); lse_g.fill_(float("nan")); ws_g.fill_(0xFF)      # nothing may survive from the last replay
        gr.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g.view(torch.int16), y_e.view(torch.int16)), rep
        assert torch.equal(lse_g.view(torch.int32), lse_e.view(torch.int32)), rep
        # eager work of the same library between the replays (other buffers)
        y2, lse2 = torch.empty_like(y_e), torch.empty_like(lse_e)
        bx.beagle_xattn_draft_step(desc, x, vc, kc, wq, wo, y2, lse2, ws)
        torch.cuda.synchronize()
    # new inputs in the same buffers: the graph reads them at replay time
    x.copy_(torch.randn(M, D, device=DEV).to(torch.bfloat16))
    bx.beagle_xattn_draft_step(desc, x, kc, vc, wq, wo, y_e, lse_e, ws)
    gr.replay()
    torch.cuda.synchronize()
    assert torch.equal(y_g.view(torch.int16), y_e.view(torch.int16))
    assert torch.equal(lse_g.view(torch.int32), lse_e.view(torch.int32))


def test_training_step_graph_replay_is_bitwise_the_eager_call():
    cfg = synth.CONFIGS["c3"].with_(batch=2, seq_q=300, seq_kv=300, hidden=512, n_q_heads=8, n_kv_heads=2)
    inp = synth.make_inputs(cfg, peaked_queries=True)
    dev, _ = gh.run_fwd_device(cfg, inp)
    g_e = gh.run_bwd_device(cfg, inp, dev)
    desc = gh.desc_of(cfg, bx.BEAGLE_FLAG_NEED_DXKV)
    dy = gh.to_dev(inp["dy"], cfg)
    outs = {n: torch.empty_like(dev[n]) for n in ("y", "lse", "q", "k", "v", "o")}
    grads = {n: torch.empty_like(t) for n, t in g_e.items()}
    ws_f, ws_b = gh.workspace(desc, bx.BEAGLE_WS_FWD), gh.workspace(desc, bx.BEAGLE_WS_BWD)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        s = torch.cuda.current_stream()
        bx.beagle_xattn_fwd(desc, dev["xq"], dev["xkv"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], outs["y"], outs["lse"],
                            outs["q"], outs["k"], outs["v"], outs["o"], ws_f, s)
        bx.beagle_xattn_bwd(desc, dy, dev["xq"], dev["xkv"], dev["wq"], dev["wk"], dev["wv"], dev["wo"], outs["q"], outs["k"],
                            outs["v"], outs["o"], outs["lse"], grads["dxq"], grads["dxkv"], grads["dwq"], grads["dwk"],
                            grads["dwv"], grads["dwo"], ws_b, s)
    for rep in range(3):
        for t in list(outs.values()) + list(grads.values()):
            t.fill_(float("nan"))
        ws_b.fill_(0xFF)
        gr.replay()
        torch.cuda.synchronize()
        for n in outs:
            assert np.array_equal(gh.to_host(outs[n]), gh.to_host(dev[n]), equal_nan=True), (rep, n)
        for n in grads:
            assert np.array_equal(gh.to_host(grads[n]), gh.to_host(g_e[n]), equal_nan=True), (rep, n)
        gh.run_fwd_device(cfg, inp)          # eager work between the replays
