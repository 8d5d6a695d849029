"""The pins are only worth something if a plausible mistake in the oracle makes one of them fail.  Each case here
plants one such mistake IN THE ORACLE (on the CPU, through monkeypatching: a wrong inequality, a dropped scale, a
flipped sign, a missing term, a forgotten residual) and checks that a named pin test then fails."""
import numpy as np
import pytest

from oracle import beagle_oracle as orc
from oracle import block_oracle as blk
import test_oracle_pins as P
import test_oracle_sim_pins as PS
import test_oracle_rope_pins as PR
import test_oracle_block_pins as PB
import test_oracle_tree_pins as PT
import test_oracle_packed_pins as PP

F64 = np.float64


def _fails(fn, *args):
    with pytest.raises((AssertionError, ValueError, IndexError)):
        fn(*args)


def test_window_hides_its_own_keys_off_by_one(monkeypatch):
    real = orc.dense_mask_loops

    def wrong(seq_q, seq_kv, k, eps=0):                     # "j <= window start" instead of "j < window start"
        m = real(seq_q, seq_kv, k, eps)
        for p in range(seq_q):
            n = int(m[p].sum())
            if n < seq_kv:
                m[p, n] = True
        return m
    monkeypatch.setattr(orc, "dense_mask_loops", wrong)
    _fails(P.test_mask_matches_handwritten_fixture, "mask_k3_eps1_s8.txt", 3, 1)
    monkeypatch.setattr(orc, "dense_mask", wrong)             # the same mistake in the closed form
    _fails(P.test_mask_k1_is_strict_causal)
    _fails(P.test_mask_visible_pair_count_closed_form, 128, 4, 7936)


def test_vectorised_mask_with_floor_division_bug(monkeypatch):
    def wrong(seq_q, seq_kv, k, eps=0):                     # truncating division: wrong for the leading partial window
        p = np.arange(seq_q)[:, None]
        j = np.arange(seq_kv)[None, :]
        ws = eps + k * ((p - eps) / k).astype(int)
        return j < np.maximum(ws, 0)
    monkeypatch.setattr(orc, "dense_mask", wrong)
    _fails(P.test_mask_vectorised_equals_loops_and_row_limit, 4)


def test_softmax_without_the_scale(monkeypatch):
    real = orc.xattn_forward

    def wrong(*a, scale=None, **kw):
        return real(*a, scale=1.0, **kw)                    # forgets 1/sqrt(d)
    monkeypatch.setattr(orc, "xattn_forward", wrong)
    _fails(P.test_forward_matches_scalar_brute_force, 2, 1, 2, 1)
    _fails(P.test_prefix_reduction_to_library_attention)


def test_mask_applied_after_normalisation(monkeypatch):
    def wrong(scores, mask):                                # Eq. 2 read literally: softmax over all keys, then mask
        s = scores - scores.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True) * mask
        with np.errstate(divide="ignore"):
            lse = np.where(mask.any(-1), np.log(np.exp(scores - scores.max(-1, keepdims=True)).sum(-1)) + scores.max(-1), -np.inf)
        return p, lse
    monkeypatch.setattr(orc, "masked_softmax", wrong)
    _fails(P.test_rows_sum_to_one_and_masked_weights_are_zero)


def test_backward_with_a_dropped_scale_on_dk(monkeypatch):
    real = orc.xattn_backward

    def wrong(*a, **kw):
        out = real(*a, **kw)
        out["dwk"] = out["dwk"] * 2.0                       # e.g. the scale applied twice on the key side
        return out
    monkeypatch.setattr(orc, "xattn_backward", wrong)
    _fails(P.test_gradients_match_central_finite_differences, 3, 1, 4, 2)
    _fails(P.test_gradients_match_autograd_float64)


def test_gqa_head_mapping_transposed(monkeypatch):
    monkeypatch.setattr(orc, "_check_heads", lambda H, G: 1 if H == G else H)   # h // rep becomes 0 for every head
    _fails(P.test_gqa_equals_mha_with_repeated_kv_heads)


def test_simulation_band_includes_the_query_itself(monkeypatch):
    real = orc.sim_pred_mask_loops

    def wrong(seq_q, seq_kv, k, eps, t):
        m = real(seq_q, seq_kv, k, eps, t)
        n = min(seq_q, seq_kv)
        for p in range(n):                                   # "j <= p" instead of "j < p", where the position holds a prediction
            w0 = eps + k * ((p - eps) // k)
            if p - w0 < t:
                m[p, p] = True
        return m
    monkeypatch.setattr(orc, "sim_pred_mask_loops", wrong)
    case = next(c for c in PS._fixtures() if c["t"] > 0)
    _fails(PS.test_pred_mask_matches_hand_written, case)


def test_save_of_predicted_states_at_the_wrong_window_position(monkeypatch):
    real = orc.sim_save_predicted
    monkeypatch.setattr(orc, "sim_save_predicted", lambda xp, h, k, eps, t: real(xp, h, k, eps, t + 1))
    _fails(PS.test_save_predicted_rows_hand_written, 10, 4, 0, 0, [0, 4, 8])
    _fails(PS.test_saved_rows_are_exactly_what_the_next_steps_may_see, 4, 0)


def test_rotary_embedding_with_a_flipped_sign(monkeypatch):
    real = orc.rope_rotate
    monkeypatch.setattr(orc, "rope_rotate", lambda x, pos, base=10000.0, inverse=False: real(x, pos, base, not inverse))
    _fails(PR.test_rotation_is_multiplication_by_a_unit_complex_number)


def test_rotary_embedding_pairing_adjacent_channels(monkeypatch):
    def wrong(x, positions, base=10000.0, inverse=False):    # (2c, 2c+1) pairs instead of (c, c + d/2)
        x = np.asarray(x, F64)
        d = x.shape[-1]
        ang = np.asarray(positions, F64)[:, None] * (float(base) ** (-2.0 * np.arange(d // 2) / d))[None, :]
        if inverse:
            ang = -ang
        cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        x1, x2 = x[..., 0::2], x[..., 1::2]
        out = np.empty_like(x)
        out[..., 0::2], out[..., 1::2] = x1 * cos - x2 * sin, x2 * cos + x1 * sin
        return out
    monkeypatch.setattr(orc, "rope_rotate", wrong)
    _fails(PR.test_rotation_is_multiplication_by_a_unit_complex_number)
    _fails(PR.test_forward_and_gradients_against_torch_autograd)


def test_rotary_gradient_not_rotated_back(monkeypatch):
    real = orc.rope_rotate
    monkeypatch.setattr(orc, "rope_rotate", lambda x, pos, base=10000.0, inverse=False: real(x, pos, base, False))
    _fails(PR.test_forward_and_gradients_against_torch_autograd)


def test_rmsnorm_backward_without_the_mean_term(monkeypatch):
    def wrong(dout, x, gain, rms_eps):
        x = np.asarray(x, F64)
        r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + rms_eps)
        return np.asarray(dout, F64) * np.asarray(gain, F64) * r, (dout * x * r).reshape(-1, x.shape[-1]).sum(0)
    monkeypatch.setattr(blk, "rmsnorm_backward", wrong)
    _fails(PB.test_rmsnorm_backward_autograd_finite_differences_and_orthogonality)
    _fails(PB.test_block_gradients_by_finite_differences)


def test_gate_and_up_swapped_and_wrong_silu_derivative(monkeypatch):
    real = blk.mlp_forward
    monkeypatch.setattr(blk, "mlp_forward", lambda z, wg, wu, wd: real(z, wu, wg, wd))
    _fails(PB.test_mlp_equals_torch_and_autograd)
    monkeypatch.setattr(blk, "mlp_forward", real)
    monkeypatch.setattr(blk, "_sigmoid", lambda u: 1.0 / (1.0 + np.exp(u)))          # sigmoid(-u)
    _fails(PB.test_silu_closed_forms)


def test_block_without_the_first_residual(monkeypatch):
    real_block = blk.block_forward

    def no_residual(e, hs, *a, **kw):
        f = real_block(e, hs, *a, **kw)
        f["h"] = f["h"] - np.asarray(e, F64)                 # forgets "+ e" (it propagates through y into h)
        return f
    monkeypatch.setattr(blk, "block_forward", no_residual)
    _fails(PB.test_the_two_residual_lines_of_eq1)
    _fails(PB.test_block_forward_and_all_gradients_against_torch, True)


def test_tree_mask_that_lets_a_node_see_itself(monkeypatch):
    real = orc.ancestor_mask

    def wrong(parents, query_nodes):
        m = real(parents, query_nodes).copy()
        for i, t in enumerate(query_nodes):
            if 0 <= t < m.shape[1]:
                m[i, t] = True
        return m
    monkeypatch.setattr(orc, "ancestor_mask", wrong)
    ran = False
    for name in dir(PT):
        if name.startswith("test_") and "hand" in name:
            fn = getattr(PT, name)
            try:
                _fails(fn)
                ran = True
            except TypeError:
                pass
    assert ran


def test_packed_sequences_that_see_their_neighbours(monkeypatch):
    real = orc.xattn_forward_packed

    def wrong(xq, xkv, wq, wk, wv, wo, cu_q, cu_kv, **kw):  # one long sequence instead of separate ones
        return real(xq, xkv, wq, wk, wv, wo, [0, cu_q[-1]], [0, cu_kv[-1]], **{**kw, "eps_list": None})
    monkeypatch.setattr(orc, "xattn_forward_packed", wrong)
    _fails(PP.test_sequences_do_not_see_each_other_and_masks_restart)
