"""Host-side checks of the C-ABI library (CPU only, no compute calls): it
loads, exports every declared symbol, its integer mask/index code agrees bit
for bit with the mask the oracle builds from the paper's prose, and invalid
arguments are rejected before anything would be launched."""
import os
import re

import numpy as np
import pytest

from oracle import beagle_oracle as orc
from paper_2505_24544_amd import binding as bx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _desc(S=16, L=None, k=4, eps=0, **kw):
    base = dict(batch=1, seq_q=S, seq_kv=S if L is None else L, hidden=256, n_q_heads=4, n_kv_heads=4,
                head_dim=64, block_size=k, block_offset=eps, io_dtype=bx.BEAGLE_F32)
    base.update(kw)
    return bx.make_desc(**base)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "beagle_xattn.h")).read()
    declared = set(re.findall(r"\b(beagle_xattn_[a-z_]+)\s*\(", hdr))
    declared.discard("beagle_xattn_desc")
    assert declared == set(bx.EXPORTS)
    L = bx.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert bx.beagle_xattn_version() == "1.0"
    assert bx.beagle_xattn_status_string(0) == "ok"
    for s in range(1, 7):
        assert bx.beagle_xattn_status_string(s) not in ("ok", "unknown status")


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8, 16])
def test_mask_and_row_limit_bit_exact_vs_oracle(k):
    for eps in sorted({0, 1, k // 2, k - 1} & set(range(k))):
        for S, L in ((1, 1), (7, 7), (64, 64), (130, 130), (257, 100), (100, 257)):
            d = _desc(S, L, k, eps)
            want = orc.dense_mask(S, L, k, eps)
            got = bx.beagle_xattn_mask_dense(d)
            assert got.dtype == np.uint8 and np.array_equal(got.astype(bool), want), (k, eps, S, L)
            lim = bx.beagle_xattn_mask_row_limit(d)
            assert np.array_equal(lim, want.sum(1).astype(np.int32))


@pytest.mark.parametrize("S,k,count", [(2048, 4, 2093056), (4096, 8, 8372224), (8192, 8, 33521664)])
def test_row_limits_at_full_size(S, k, count):
    lim = bx.beagle_xattn_mask_row_limit(_desc(S, S, k, 0))
    assert int(lim.astype(np.int64).sum()) == count
    assert np.array_equal(lim, orc.dense_mask(S, S, k, 0).sum(1).astype(np.int32))


@pytest.mark.parametrize("tq,tk", [(128, 64), (64, 64), (32, 16), (128, 128), (48, 20)])
def test_tile_classes_vs_oracle_mask(tq, tk):
    for (S, L, k, eps) in ((300, 300, 4, 0), (512, 512, 8, 3), (257, 190, 5, 2), (130, 400, 1, 0), (64, 64, 3, 1)):
        cls = bx.beagle_xattn_tile_map(_desc(S, L, k, eps), tq, tk)
        m = orc.dense_mask(S, L, k, eps)
        assert cls.shape == (-(-S // tq), -(-L // tk))
        for a in range(cls.shape[0]):
            for c in range(cls.shape[1]):
                blk = m[a * tq:(a + 1) * tq, c * tk:(c + 1) * tk]
                want = 0 if not blk.any() else (2 if blk.all() else 1)
                assert cls[a, c] == want, (S, L, k, eps, a, c)


def test_skipped_tile_fraction_matches_block_structure():
    # 128x128 tiles on the 7B-shaped config: 120 full, 16 partial, 120 skipped
    cls = bx.beagle_xattn_tile_map(_desc(2048, 2048, 4, 0), 128, 128)
    assert [(cls == v).sum() for v in (2, 1, 0)] == [120, 16, 120]


def test_invalid_descriptors_are_rejected_on_the_host():
    E = bx.BeagleError
    bad = [dict(k=0), dict(k=4, eps=4), dict(eps=-1), dict(S=0), dict(n_kv_heads=3), dict(head_dim=0),
           dict(io_dtype=7), dict(flags=1 << 9), dict(softmax_scale=-1.0), dict(batch=0)]
    for kw in bad:
        with pytest.raises(E):
            bx.beagle_xattn_mask_row_limit(_desc(**kw))
        assert bx.beagle_xattn_workspace_bytes(_desc(**kw), bx.BEAGLE_WS_BWD) == 0
    d = _desc()
    d.struct_size = 8
    with pytest.raises(E) as ei:
        bx.beagle_xattn_mask_row_limit(d)
    assert ei.value.status == 2
    # unsupported shapes: bf16 needs d == 128 and D % 64 == 0; f32 needs d <= 128
    for kw in (dict(io_dtype=bx.BEAGLE_BF16, head_dim=64), dict(io_dtype=bx.BEAGLE_BF16, head_dim=128, hidden=200),
               dict(head_dim=256), dict(head_dim=6)):
        with pytest.raises(E) as ei:
            bx.beagle_xattn_mask_row_limit(_desc(**kw))
        assert ei.value.status == 3
    with pytest.raises(E):
        bx.beagle_xattn_tile_map(_desc(), 0, 4)
    # window sizes and lengths beyond 2^30 would overflow the int32 index code
    for kw in (dict(k=2 ** 30 + 1), dict(S=2 ** 30 + 1, L=4), dict(S=4, L=2 ** 30 + 1)):
        assert bx.beagle_xattn_workspace_bytes(_desc(**kw), bx.BEAGLE_WS_FWD) == 0
    assert bx.beagle_xattn_workspace_bytes(_desc(k=2 ** 30), bx.BEAGLE_WS_FWD) > 0
    # bf16: one batch entry's K/V slab must stay below 2 GiB (32-bit buffer descriptors)
    big = dict(io_dtype=bx.BEAGLE_BF16, head_dim=128, hidden=4096, n_q_heads=32, n_kv_heads=32)
    assert bx.beagle_xattn_workspace_bytes(_desc(S=262143, **big), bx.BEAGLE_WS_FWD) > 0
    assert bx.beagle_xattn_workspace_bytes(_desc(S=262144, **big), bx.BEAGLE_WS_FWD) == 0


def test_projection_operands_of_2_gib_are_refused_not_rerouted():
    """bf16: every operand of the projection kernels is addressed through a 32-bit buffer descriptor; a batch whose
    activations reach 2 GiB (B*S*D*2 bytes) is refused with BEAGLE_ERR_UNSUPPORTED before anything is enqueued --
    there is no slower kernel it could be sent to."""
    a, ws = 4096, 1 << 62
    big = dict(io_dtype=bx.BEAGLE_BF16, head_dim=128, hidden=4096, n_q_heads=32, n_kv_heads=32, k=4)
    ok = _desc(S=2048, batch=127, **big)            # 127 * 2048 * 4096 * 2 < 2^31
    no = _desc(S=2048, batch=128, **big)            # exactly 2^31
    assert bx.beagle_xattn_workspace_bytes(ok, bx.BEAGLE_WS_BWD) > 0
    assert bx.beagle_xattn_workspace_bytes(no, bx.BEAGLE_WS_BWD) == 0
    assert bx.beagle_xattn_fwd(no, *([a] * 12), a, stream=0, workspace_bytes=ws, check=False) == 3
    assert bx.beagle_xattn_bwd(no, *([a] * 18), a, stream=0, workspace_bytes=ws, check=False) == 3
    # S != L: the longer side decides; GQA: the query side's H*d decides
    assert bx.beagle_xattn_workspace_bytes(_desc(S=16, L=262144, **big), bx.BEAGLE_WS_FWD) == 0
    gqa = dict(big, n_kv_heads=8)
    assert bx.beagle_xattn_workspace_bytes(_desc(S=2048, batch=128, **gqa), bx.BEAGLE_WS_FWD) == 0
    # packed batches: the packed row count decides, not batch * longest
    pk = dict(big, cu_seqlens_q=a, cu_seqlens_kv=a)
    assert bx.beagle_xattn_workspace_bytes(_desc(S=2048, batch=200, total_q=200000, total_kv=200000, **pk), bx.BEAGLE_WS_FWD) > 0
    assert bx.beagle_xattn_workspace_bytes(_desc(S=2048, batch=200, total_q=262144, total_kv=200000, **pk), bx.BEAGLE_WS_FWD) == 0
    # a weight matrix of 2 GiB
    wide = dict(io_dtype=bx.BEAGLE_BF16, head_dim=128, hidden=32768, n_q_heads=256, n_kv_heads=256, k=4)
    assert bx.beagle_xattn_workspace_bytes(_desc(S=16, **wide), bx.BEAGLE_WS_FWD) == 0
    # the feed-forward operands of the block entry points
    assert bx.beagle_xattn_block_workspace_bytes(ok, 4096, bx.BEAGLE_WS_BLOCK_BWD) > 0
    prm = bx.make_block_params(8192, 1e-5, **{n: a for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")})
    sv = bx.make_block_saved(**{n: a for n in ("q", "k", "v", "o", "lse", "y", "u", "w", "m")})
    assert bx.beagle_xattn_block_fwd(ok, prm, a, a, a, sv, a, stream=0, workspace_bytes=ws, check=False) == 3


def test_tree_and_append_entry_points_validate_before_launching():
    d = _desc(S=4, L=100)
    a = 4096
    ws = 1 << 30
    tree = lambda n_true, mask, words: bx.beagle_xattn_draft_step_tree(
        d, a, a, a, a, a, n_true, mask, words, a, a, a, stream=0, workspace_bytes=ws, check=False)
    assert tree(101, a, 4) == 2 and tree(-1, a, 4) == 2          # n_true outside [0, L]
    assert tree(50, None, 2) == 1                                 # drafted rows but no mask
    assert tree(50, a, 1) == 2                                    # 50 drafted rows need 2 words
    assert tree(50, a + 2, 2) == 5                                # mask not 4-byte aligned
    app = lambda pos, wsb=ws: bx.beagle_xattn_kv_append(d, a, a, a, a, a, pos, a, stream=0, workspace_bytes=wsb,
                                                        check=False)
    assert app(97) == 2 and app(-1) == 2                          # rows pos .. pos+3 must fit in 100
    assert app(0, 8) == 4
    assert bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_APPEND) > 0


def test_simulation_entry_points_validate_before_launching():
    a, ws = 4096, 1 << 40
    d = _desc(S=64, L=64)
    fwd = lambda dd, t, xp=a: bx.beagle_xattn_fwd_sim(dd, a, a, xp, a, a, a, a, t, a, a, a, a, a, a, a, a, a, stream=0,
                                                      workspace_bytes=ws, check=False)
    assert fwd(_desc(S=32, L=64), 1) == 2                       # needs seq_q == seq_kv
    assert fwd(d, -1) == 2 and fwd(d, 1, None) == 1 and fwd(d, 1, a + 8) == 5
    bwd = lambda dd, t, dxp=a, wsb=ws: bx.beagle_xattn_bwd_sim(dd, *([a] * 15), t, a, a, dxp, a, a, a, a, a, stream=0,
                                                               workspace_bytes=wsb, check=False)
    assert bwd(_desc(S=32, L=64), 1) == 2 and bwd(d, -1) == 2
    assert bwd(d, 1, None) == 1                                 # the buffer's gradient is a required output
    assert bwd(d, 1, a, 64) == 4
    assert bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_BWD_SIM) > bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_BWD)
    save = lambda dd, t, h=a: bx.beagle_xattn_sim_save(dd, h, a, t, stream=0, check=False)
    assert save(_desc(S=32, L=64), 0) == 2 and save(d, -1) == 2 and save(d, 0, None) == 1 and save(d, 0, a + 4) == 5


def test_block_entry_points_validate_before_launching():
    a = 4096
    d = _desc(S=16, L=16)
    W = dict(wq=a, wk=a, wv=a, wo=a, w_gate=a, w_up=a, w_down=a)
    sv = bx.make_block_saved(**{n: a for n in ("q", "k", "v", "o", "lse", "y", "u", "w", "m")})
    fwd = lambda p, s=sv, e=a: bx.beagle_xattn_block_fwd(d, p, e, a, a, s, None, stream=0, check=False)
    assert fwd(bx.make_block_params(30, 1e-5, **W)) == 3                 # F % 4 != 0
    assert fwd(bx.make_block_params(0, 1e-5, **W)) == 2
    assert fwd(bx.make_block_params(32, float("nan"), **W)) == 2
    assert fwd(bx.make_block_params(32, 1e-5, **dict(W, w_down=None))) == 1
    assert fwd(bx.make_block_params(32, 1e-5, g_mlp=a, **W)) == 1         # gain without z / r_mlp
    assert fwd(bx.make_block_params(32, 1e-5, **W), None) == 1
    assert fwd(bx.make_block_params(32, 1e-5, **W), sv, a + 4) == 5
    bad = bx.make_block_params(32, 1e-5, **W)
    bad.struct_size = 8
    assert fwd(bad) == 2
    gr = bx.make_block_grads(**{n: a for n in ("de", "dwq", "dwk", "dwv", "dwo", "dw_gate", "dw_up", "dw_down")})
    ok = bx.make_block_params(32, 1e-5, **W)
    bwd = lambda g, wsb: bx.beagle_xattn_block_bwd(d, ok, a, a, a, sv, g, a, stream=0, workspace_bytes=wsb, check=False)
    assert bwd(gr, 64) == 4 and bwd(None, 1 << 40) == 1
    assert bx.beagle_xattn_block_bwd(_desc(S=16, L=16, flags=bx.BEAGLE_FLAG_NEED_DXKV), ok, a, a, a, sv, gr, a, stream=0,
                                     workspace_bytes=1 << 40, check=False) == 1   # dhs requested but not given
    assert bx.beagle_xattn_block_bwd(_desc(S=16, L=16, flags=bx.BEAGLE_FLAG_WGRAD_F32), ok, a, a, a, sv, gr, a, stream=0,
                                     workspace_bytes=1 << 40, check=False) == 3
    n = bx.beagle_xattn_block_workspace_bytes(d, 32, bx.BEAGLE_WS_BLOCK_BWD)
    assert n > bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_BWD) and bx.beagle_xattn_block_workspace_bytes(d, 30, 1) == 0
    with pytest.raises(KeyError):
        bx.make_block_saved(nonsense=a)


def test_block_simulation_and_decode_entry_points_validate_before_launching():
    a, big = 4096, 1 << 40
    d = _desc(S=16, L=16)
    W = dict(wq=a, wk=a, wv=a, wo=a, w_gate=a, w_up=a, w_down=a)
    base = {n: a for n in ("q", "k", "v", "o", "lse", "y", "u", "w", "m")}
    ok = bx.make_block_params(32, 1e-5, **W)
    fwd = lambda sv, xp=a, t=1, dd=d: bx.beagle_xattn_block_fwd_sim(dd, ok, a, a, xp, t, a, bx.make_block_saved(**sv), None,
                                                                    stream=0, check=False)
    assert fwd(base) == 1                                          # kp / vp missing
    full = dict(base, kp=a, vp=a)
    assert fwd(full, None) == 1 and fwd(full, a, -1) == 2 and fwd(full, a, 1, _desc(S=8, L=16)) == 2
    withg = bx.make_block_params(32, 1e-5, g_kv=a, **W)
    sv_g = bx.make_block_saved(**dict(full, xkv_n=a, r_kv=a))       # gain given, but no room for the normalised xpred
    assert bx.beagle_xattn_block_fwd_sim(d, withg, a, a, a, 1, a, sv_g, None, stream=0, check=False) == 1
    gr = {n: a for n in ("de", "dwq", "dwk", "dwv", "dwo", "dw_gate", "dw_up", "dw_down")}
    bwd = lambda g, wsb=big: bx.beagle_xattn_block_bwd_sim(d, ok, a, a, a, a, 1, bx.make_block_saved(**full),
                                                           bx.make_block_grads(**g), a, stream=0, workspace_bytes=wsb, check=False)
    assert bwd(gr) == 1                                            # dxpred is a required output
    assert bwd(dict(gr, dxpred=a), 64) == 4
    n_sim = bx.beagle_xattn_block_workspace_bytes(d, 32, bx.BEAGLE_WS_BLOCK_BWD_SIM)
    assert n_sim > bx.beagle_xattn_block_workspace_bytes(d, 32, bx.BEAGLE_WS_BLOCK_BWD)
    # decode-time block
    dd = _desc(S=2, L=16)
    step = lambda p, n_true=16, wsb=big: bx.beagle_xattn_block_draft_step(dd, p, a, a, a, n_true, None, 0, a, a, a, stream=0,
                                                                         workspace_bytes=wsb, check=False)
    dW = dict(wq=a, wo=a, w_gate=a, w_up=a, w_down=a)              # wk, wv, g_kv are not needed at decode time
    assert step(bx.make_block_params(32, 1e-5, **dict(dW, w_gate=None))) == 1
    assert step(bx.make_block_params(32, 1e-5, **dW), 17) == 2 and step(bx.make_block_params(32, 1e-5, **dW), 10) == 1
    assert step(bx.make_block_params(32, 1e-5, **dW), 16, 64) == 4
    assert bx.beagle_xattn_block_workspace_bytes(dd, 32, bx.BEAGLE_WS_BLOCK_DRAFT) > 0
    assert bx.beagle_xattn_block_workspace_bytes(_desc(S=2, L=16, batch=2), 32, bx.BEAGLE_WS_BLOCK_DRAFT) == 0


def test_entry_points_validate_before_launching():
    """NULL / misaligned / short-workspace arguments return a status without
    touching the GPU (this test runs where there is none)."""
    d = _desc()
    a = 4096  # fake, aligned, never dereferenced: validation fails first
    st = bx.beagle_xattn_fwd(d, a, a, a, a, a, a, a, a, a, a, a, None, None, stream=0, check=False)
    assert st == 1
    st = bx.beagle_xattn_fwd(d, a, a, a, a + 4, a, a, a, a, a, a, a, a, None, stream=0, check=False)
    assert st == 5
    args = [a] * 18
    st = bx.beagle_xattn_bwd(d, *args, None, stream=0, check=False)
    assert st == 1
    st = bx.beagle_xattn_bwd(d, *args, a, stream=0, workspace_bytes=16, check=False)
    assert st == 4
    d2 = _desc(flags=bx.BEAGLE_FLAG_NEED_DXKV)
    args[13] = None
    assert bx.beagle_xattn_bwd(d2, *args, a, stream=0, workspace_bytes=1 << 30, check=False) == 1
    assert bx.beagle_xattn_draft_step(_desc(batch=2), a, a, a, a, a, a, a, a, stream=0, workspace_bytes=1 << 30,
                                      check=False) == 2
    assert bx.beagle_xattn_draft_step(d, a, a, a, a, a, a, a, a, stream=0, workspace_bytes=8, check=False) == 4
    assert bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_BWD) > 0
    assert bx.beagle_xattn_workspace_bytes(d, 99) == 0


def test_workspace_is_linear_in_sequence_length():
    """Constant-space masks: no S x L buffer anywhere in the workspace."""
    def ws(S):
        d = bx.make_desc(batch=1, seq_q=S, seq_kv=S, hidden=4096, n_q_heads=32, n_kv_heads=32, head_dim=128,
                         block_size=4, io_dtype=bx.BEAGLE_BF16, flags=bx.BEAGLE_FLAG_NEED_DXKV)
        return bx.beagle_xattn_workspace_bytes(d, bx.BEAGLE_WS_BWD)
    a, b, c = ws(1024), ws(2048), ws(4096)
    assert abs((c - b) - 2 * (b - a)) <= 4096 and c < 3 * b
