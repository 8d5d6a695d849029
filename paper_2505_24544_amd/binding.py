"""ctypes binding over libbeagle_xattn.so: argument marshalling only.

Function names mirror include/beagle_xattn.h.  Tensor arguments may be torch
tensors (their data_ptr() is passed; they must be contiguous) or raw integer
device addresses.  PyTorch is used for device allocations and streams only;
every step of the computation runs inside the library's kernels.  There is no
fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbeagle_xattn.so")

BEAGLE_OK = 0
(BEAGLE_ERR_NULL, BEAGLE_ERR_SHAPE, BEAGLE_ERR_UNSUPPORTED, BEAGLE_ERR_WORKSPACE, BEAGLE_ERR_ALIGN,
 BEAGLE_ERR_HIP) = range(1, 7)
BEAGLE_F32, BEAGLE_BF16 = 0, 1
BEAGLE_FLAG_NEED_DXKV, BEAGLE_FLAG_WGRAD_F32, BEAGLE_FLAG_ROPE, BEAGLE_FLAG_STATES_F16 = 1, 2, 4, 8
BEAGLE_WS_FWD, BEAGLE_WS_BWD, BEAGLE_WS_DRAFT, BEAGLE_WS_APPEND, BEAGLE_WS_BWD_SIM, BEAGLE_WS_BLOCK_APPEND = 0, 1, 2, 3, 4, 5
BEAGLE_WS_BLOCK_FWD, BEAGLE_WS_BLOCK_BWD, BEAGLE_WS_BLOCK_DRAFT, BEAGLE_WS_BLOCK_BWD_SIM = 0, 1, 2, 3
STATUS_NAMES = {0: "BEAGLE_OK", 1: "BEAGLE_ERR_NULL", 2: "BEAGLE_ERR_SHAPE", 3: "BEAGLE_ERR_UNSUPPORTED",
                4: "BEAGLE_ERR_WORKSPACE", 5: "BEAGLE_ERR_ALIGN", 6: "BEAGLE_ERR_HIP"}

EXPORTS = (
    "beagle_xattn_workspace_bytes", "beagle_xattn_fwd", "beagle_xattn_bwd", "beagle_xattn_draft_step",
    "beagle_xattn_draft_step_static", "beagle_xattn_draft_step_tree", "beagle_xattn_prepare_weights", "beagle_xattn_kv_append_prepared", "beagle_xattn_block_kv_append_prepared",
    "beagle_xattn_draft_step_prepared", "beagle_xattn_kv_append", "beagle_xattn_fwd_sim", "beagle_xattn_bwd_sim",
    "beagle_xattn_sim_save",
    "beagle_xattn_block_workspace_bytes", "beagle_xattn_block_fwd", "beagle_xattn_block_bwd",
    "beagle_xattn_block_draft_step", "beagle_xattn_block_draft_step_prepared", "beagle_xattn_block_prepare_weights",
    "beagle_xattn_block_fwd_sim", "beagle_xattn_block_bwd_sim",
    "beagle_xattn_block_kv_append",
    "beagle_xattn_mask_row_limit", "beagle_xattn_mask_dense", "beagle_xattn_tile_map",
    "beagle_xattn_profile_begin", "beagle_xattn_profile_end", "beagle_xattn_profile_get",
    "beagle_xattn_probe_read", "beagle_xattn_probe_clock", "beagle_xattn_status_string", "beagle_xattn_version",
)


class BeagleError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, STATUS_NAMES.get(status, "?"), status))


class beagle_xattn_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_int32), ("batch", C.c_int32), ("seq_q", C.c_int32), ("seq_kv", C.c_int32),
        ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("block_size", C.c_int32), ("block_offset", C.c_int32), ("io_dtype", C.c_int32),
        ("softmax_scale", C.c_float), ("flags", C.c_uint32), ("block_offsets", C.c_void_p),
        ("cu_seqlens_q", C.c_void_p), ("cu_seqlens_kv", C.c_void_p), ("total_q", C.c_int32), ("total_kv", C.c_int32),
        ("rope_base", C.c_float), ("rope_positions", C.c_void_p),
    ]


def make_desc(*, batch, seq_q, seq_kv, hidden, n_q_heads, n_kv_heads, head_dim, block_size=1,
              block_offset=0, io_dtype=BEAGLE_BF16, softmax_scale=0.0, flags=0,
              block_offsets=None, rope_base=0.0, rope_positions=None, cu_seqlens_q=None, cu_seqlens_kv=None,
              total_q=0, total_kv=0) -> beagle_xattn_desc:
    """block_offsets: None, or an int32 device tensor / address of B per-entry offsets (kept alive by the caller)."""
    return beagle_xattn_desc(C.sizeof(beagle_xattn_desc), batch, seq_q, seq_kv, hidden, n_q_heads, n_kv_heads,
                             head_dim, block_size, block_offset, io_dtype, softmax_scale, flags, _ptr(block_offsets),
                             _ptr(cu_seqlens_q), _ptr(cu_seqlens_kv), total_q, total_kv, rope_base, _ptr(rope_positions))


_VP = C.c_void_p


class beagle_block_params(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("ffn", C.c_int32), ("rms_eps", C.c_float), ("reserved", C.c_int32)] + \
               [(n, _VP) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_q", "g_kv", "g_mlp")]


class beagle_block_decode_weights(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("reserved", C.c_int32)] + \
               [(n, _VP) for n in ("wq_pk", "wo_pk", "wk_pk", "wv_pk", "w_gate_pk", "w_up_pk", "w_down_pk")]


class beagle_block_saved(C.Structure):
    _fields_ = [(n, _VP) for n in ("xq_n", "r_q", "xkv_n", "r_kv", "q", "k", "v", "o", "lse", "y", "z", "r_mlp",
                                   "u", "w", "m", "xp_n", "r_p", "kp", "vp")]


class beagle_block_grads(C.Structure):
    _fields_ = [(n, _VP) for n in ("de", "dhs", "dwq", "dwk", "dwv", "dwo", "dw_gate", "dw_up", "dw_down",
                                   "dg_q", "dg_kv", "dg_mlp", "dxpred")]


def _fill(struct, tensors: dict):
    """Pointer struct from a dict name -> tensor / address / None; keeps nothing alive (the caller does)."""
    names = [f[0] for f in struct._fields_ if f[1] is _VP]
    unknown = set(tensors) - set(names)
    if unknown:
        raise KeyError("unknown field(s): %s" % sorted(unknown))
    out = struct()
    for n in names:
        setattr(out, n, _ptr(tensors.get(n)))
    return out


def make_block_params(ffn, rms_eps, **weights) -> beagle_block_params:
    p = _fill(beagle_block_params, weights)
    p.struct_size, p.ffn, p.rms_eps, p.reserved = C.sizeof(beagle_block_params), int(ffn), float(rms_eps), 0
    return p


def make_block_decode_weights(**tensors) -> beagle_block_decode_weights:
    w = _fill(beagle_block_decode_weights, tensors)
    w.struct_size, w.reserved = C.sizeof(beagle_block_decode_weights), 0
    return w


def make_block_saved(**tensors) -> beagle_block_saved:
    return _fill(beagle_block_saved, tensors)


def make_block_grads(**tensors) -> beagle_block_grads:
    return _fill(beagle_block_grads, tensors)


_lib = None


def lib() -> C.CDLL:
    """Open the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s not found: build it with `python -m paper_2505_24544_amd.build` "
                           "(there is no fallback path)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, dp = C.c_void_p, C.POINTER(beagle_xattn_desc)
    L.beagle_xattn_workspace_bytes.restype = C.c_size_t
    L.beagle_xattn_workspace_bytes.argtypes = [dp, C.c_int]
    L.beagle_xattn_fwd.restype = C.c_int
    L.beagle_xattn_fwd.argtypes = [dp] + [vp] * 12 + [vp, C.c_size_t, vp]
    L.beagle_xattn_bwd.restype = C.c_int
    L.beagle_xattn_bwd.argtypes = [dp] + [vp] * 18 + [vp, C.c_size_t, vp]
    L.beagle_xattn_draft_step.restype = C.c_int
    L.beagle_xattn_draft_step.argtypes = [dp] + [vp] * 7 + [vp, C.c_size_t, vp]
    L.beagle_xattn_draft_step_static.restype = C.c_int
    L.beagle_xattn_draft_step_static.argtypes = [dp] + [vp] * 7 + [vp]
    L.beagle_xattn_fwd_sim.restype = C.c_int
    L.beagle_xattn_fwd_sim.argtypes = [dp] + [vp] * 7 + [C.c_int32] + [vp] * 8 + [vp, C.c_size_t, vp]
    L.beagle_xattn_bwd_sim.restype = C.c_int
    L.beagle_xattn_bwd_sim.argtypes = [dp] + [vp] * 15 + [C.c_int32] + [vp] * 7 + [vp, C.c_size_t, vp]
    L.beagle_xattn_sim_save.restype = C.c_int
    L.beagle_xattn_sim_save.argtypes = [dp, vp, vp, C.c_int32, vp]
    L.beagle_xattn_block_workspace_bytes.restype = C.c_size_t
    L.beagle_xattn_block_workspace_bytes.argtypes = [dp, C.c_int32, C.c_int]
    L.beagle_xattn_block_fwd.restype = C.c_int
    L.beagle_xattn_block_fwd.argtypes = [dp, C.POINTER(beagle_block_params), vp, vp, vp, C.POINTER(beagle_block_saved),
                                         vp, C.c_size_t, vp]
    L.beagle_xattn_block_bwd.restype = C.c_int
    L.beagle_xattn_block_bwd.argtypes = [dp, C.POINTER(beagle_block_params), vp, vp, vp, C.POINTER(beagle_block_saved),
                                         C.POINTER(beagle_block_grads), vp, C.c_size_t, vp]
    L.beagle_xattn_block_fwd_sim.restype = C.c_int
    L.beagle_xattn_block_fwd_sim.argtypes = [dp, C.POINTER(beagle_block_params), vp, vp, vp, C.c_int32, vp,
                                             C.POINTER(beagle_block_saved), vp, C.c_size_t, vp]
    L.beagle_xattn_block_bwd_sim.restype = C.c_int
    L.beagle_xattn_block_bwd_sim.argtypes = [dp, C.POINTER(beagle_block_params), vp, vp, vp, vp, C.c_int32,
                                             C.POINTER(beagle_block_saved), C.POINTER(beagle_block_grads), vp, C.c_size_t, vp]
    L.beagle_xattn_block_kv_append.restype = C.c_int
    L.beagle_xattn_block_kv_append.argtypes = [dp, C.POINTER(beagle_block_params), vp, vp, vp, C.c_int32, vp, C.c_size_t, vp]
    L.beagle_xattn_block_draft_step_prepared.restype = C.c_int
    L.beagle_xattn_block_draft_step_prepared.argtypes = [dp, C.POINTER(beagle_block_params), C.POINTER(beagle_block_decode_weights),
                                                         vp, vp, vp, C.c_int32, vp, C.c_int32, vp, vp, vp, C.c_size_t, vp]
    L.beagle_xattn_block_prepare_weights.restype = C.c_int
    L.beagle_xattn_block_prepare_weights.argtypes = [dp, C.POINTER(beagle_block_params), C.POINTER(beagle_block_decode_weights), vp]
    L.beagle_xattn_block_draft_step.restype = C.c_int
    L.beagle_xattn_block_draft_step.argtypes = [dp, C.POINTER(beagle_block_params), vp, vp, vp, C.c_int32, vp, C.c_int32,
                                                vp, vp, vp, C.c_size_t, vp]
    L.beagle_xattn_draft_step_tree.restype = C.c_int
    L.beagle_xattn_draft_step_tree.argtypes = [dp] + [vp] * 5 + [C.c_int32, vp, C.c_int32, vp, vp, vp, C.c_size_t, vp]
    L.beagle_xattn_draft_step_prepared.restype = C.c_int
    L.beagle_xattn_draft_step_prepared.argtypes = [dp] + [vp] * 5 + [C.c_int32, vp, C.c_int32, vp, vp, vp, C.c_size_t, vp]
    L.beagle_xattn_prepare_weights.restype = C.c_int
    L.beagle_xattn_prepare_weights.argtypes = [dp] + [vp] * 9
    L.beagle_xattn_kv_append_prepared.restype = C.c_int
    L.beagle_xattn_kv_append_prepared.argtypes = [dp, vp, vp, vp, vp, vp, C.c_int32, vp]
    L.beagle_xattn_block_kv_append_prepared.restype = C.c_int
    L.beagle_xattn_block_kv_append_prepared.argtypes = [dp, C.POINTER(beagle_block_params), C.POINTER(beagle_block_decode_weights),
                                                        vp, vp, vp, C.c_int32, vp]
    L.beagle_xattn_kv_append.restype = C.c_int
    L.beagle_xattn_kv_append.argtypes = [dp] + [vp] * 5 + [C.c_int32, vp, C.c_size_t, vp]
    L.beagle_xattn_mask_row_limit.restype = C.c_int
    L.beagle_xattn_mask_row_limit.argtypes = [dp, vp]
    L.beagle_xattn_mask_dense.restype = C.c_int
    L.beagle_xattn_mask_dense.argtypes = [dp, vp]
    L.beagle_xattn_tile_map.restype = C.c_int
    L.beagle_xattn_tile_map.argtypes = [dp, C.c_int32, C.c_int32, vp]
    L.beagle_xattn_profile_begin.restype = C.c_int
    L.beagle_xattn_profile_begin.argtypes = []
    L.beagle_xattn_profile_end.restype = C.c_int32
    L.beagle_xattn_profile_end.argtypes = []
    L.beagle_xattn_profile_get.restype = C.c_int
    L.beagle_xattn_profile_get.argtypes = [C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_int32),
                                           C.POINTER(C.c_double)]
    L.beagle_xattn_probe_read.restype = C.c_int
    L.beagle_xattn_probe_read.argtypes = [vp, C.c_size_t, C.c_int32, vp, vp]
    L.beagle_xattn_probe_clock.restype = C.c_int
    L.beagle_xattn_probe_clock.argtypes = [vp, vp]
    L.beagle_xattn_status_string.restype = C.c_char_p
    L.beagle_xattn_status_string.argtypes = [C.c_int]
    L.beagle_xattn_version.restype = C.c_char_p
    L.beagle_xattn_version.argtypes = []
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor arguments must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _nbytes(ws):
    if ws is None:
        return 0
    return ws.numel() * ws.element_size()


def _check(st, where, check):
    if check and st != BEAGLE_OK:
        raise BeagleError(st, where)
    return st


def beagle_xattn_fwd_sim(desc, xq, xkv, xpred, wq, wk, wv, wo, sim_step, y, lse, q_save, k_save, v_save,
                         kp_save, vp_save, o_save, workspace=None, stream=None, *, workspace_bytes=None,
                         check=True) -> int:
    st = lib().beagle_xattn_fwd_sim(
        C.byref(desc), *(_ptr(t) for t in (xq, xkv, xpred, wq, wk, wv, wo)), int(sim_step),
        *(_ptr(t) for t in (y, lse, q_save, k_save, v_save, kp_save, vp_save, o_save)),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_fwd_sim", check)


def beagle_xattn_bwd_sim(desc, dy, xq, xkv, xpred, wq, wk, wv, wo, q_save, k_save, v_save, kp_save, vp_save,
                         o_save, lse, sim_step, dxq, dxkv, dxpred, dwq, dwk, dwv, dwo, workspace, stream=None, *,
                         workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_bwd_sim(
        C.byref(desc), *(_ptr(t) for t in (dy, xq, xkv, xpred, wq, wk, wv, wo, q_save, k_save, v_save, kp_save,
                                           vp_save, o_save, lse)), int(sim_step),
        *(_ptr(t) for t in (dxq, dxkv, dxpred, dwq, dwk, dwv, dwo)),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_bwd_sim", check)


def beagle_xattn_block_workspace_bytes(desc, ffn, which) -> int:
    return int(lib().beagle_xattn_block_workspace_bytes(C.byref(desc), int(ffn), int(which)))


def beagle_xattn_block_fwd(desc, params, e, hs, h, saved, workspace=None, stream=None, *, workspace_bytes=None,
                           check=True) -> int:
    st = lib().beagle_xattn_block_fwd(
        C.byref(desc), C.byref(params) if params is not None else None, _ptr(e), _ptr(hs), _ptr(h),
        C.byref(saved) if saved is not None else None,
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_block_fwd", check)


def beagle_xattn_block_bwd(desc, params, dh, e, hs, saved, grads, workspace, stream=None, *, workspace_bytes=None,
                           check=True) -> int:
    st = lib().beagle_xattn_block_bwd(
        C.byref(desc), C.byref(params) if params is not None else None, _ptr(dh), _ptr(e), _ptr(hs),
        C.byref(saved) if saved is not None else None, C.byref(grads) if grads is not None else None,
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_block_bwd", check)


def beagle_xattn_block_fwd_sim(desc, params, e, hs, xpred, sim_step, h, saved, workspace=None, stream=None, *,
                               workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_block_fwd_sim(
        C.byref(desc), C.byref(params), _ptr(e), _ptr(hs), _ptr(xpred), int(sim_step), _ptr(h), C.byref(saved),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_block_fwd_sim", check)


def beagle_xattn_block_bwd_sim(desc, params, dh, e, hs, xpred, sim_step, saved, grads, workspace, stream=None, *,
                               workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_block_bwd_sim(
        C.byref(desc), C.byref(params), _ptr(dh), _ptr(e), _ptr(hs), _ptr(xpred), int(sim_step), C.byref(saved),
        C.byref(grads), _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes,
        _stream(stream))
    return _check(st, "beagle_xattn_block_bwd_sim", check)


def beagle_xattn_block_kv_append(desc, params, x_new, k_cache, v_cache, pos, workspace, stream=None, *,
                                 workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_block_kv_append(
        C.byref(desc), C.byref(params) if params is not None else None, _ptr(x_new), _ptr(k_cache), _ptr(v_cache), int(pos),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_block_kv_append", check)


def beagle_xattn_block_draft_step(desc, params, x_draft, k_cache, v_cache, n_true, tree_mask, mask_words, h, lse,
                                  workspace, stream=None, *, workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_block_draft_step(
        C.byref(desc), C.byref(params) if params is not None else None, _ptr(x_draft), _ptr(k_cache), _ptr(v_cache),
        int(n_true), _ptr(tree_mask), int(mask_words), _ptr(h), _ptr(lse),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_block_draft_step", check)


def beagle_xattn_block_prepare_weights(desc, params, dw, stream=None, *, check=True) -> int:
    st = lib().beagle_xattn_block_prepare_weights(C.byref(desc), C.byref(params) if params is not None else None,
                                                  C.byref(dw) if dw is not None else None, _stream(stream))
    return _check(st, "beagle_xattn_block_prepare_weights", check)


def beagle_xattn_block_draft_step_prepared(desc, params, dw, x_draft, k_cache, v_cache, n_true, tree_mask, mask_words,
                                           h, lse, workspace, stream=None, *, workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_block_draft_step_prepared(
        C.byref(desc), C.byref(params) if params is not None else None, C.byref(dw) if dw is not None else None,
        _ptr(x_draft), _ptr(k_cache), _ptr(v_cache), int(n_true), _ptr(tree_mask), int(mask_words), _ptr(h), _ptr(lse),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_block_draft_step_prepared", check)


def beagle_xattn_sim_save(desc, h, xpred, sim_step, stream=None, *, check=True) -> int:
    st = lib().beagle_xattn_sim_save(C.byref(desc), _ptr(h), _ptr(xpred), int(sim_step), _stream(stream))
    return _check(st, "beagle_xattn_sim_save", check)


def beagle_xattn_draft_step_tree(desc, x_draft, k_cache, v_cache, wq, wo, n_true, tree_mask, mask_words, y, lse,
                                 workspace, stream=None, *, workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_draft_step_tree(
        C.byref(desc), *(_ptr(t) for t in (x_draft, k_cache, v_cache, wq, wo)), int(n_true), _ptr(tree_mask),
        int(mask_words), _ptr(y), _ptr(lse),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_draft_step_tree", check)


def beagle_xattn_prepare_weights(desc, wq=None, wk=None, wv=None, wo=None, wq_pk=None, wk_pk=None, wv_pk=None, wo_pk=None,
                                 stream=None, *, check=True) -> int:
    st = lib().beagle_xattn_prepare_weights(C.byref(desc), *(_ptr(t) for t in (wq, wk, wv, wo, wq_pk, wk_pk, wv_pk, wo_pk)),
                                            _stream(stream))
    return _check(st, "beagle_xattn_prepare_weights", check)


def beagle_xattn_kv_append_prepared(desc, x_new, wk_pk, wv_pk, k_cache, v_cache, pos, stream=None, *, check=True) -> int:
    st = lib().beagle_xattn_kv_append_prepared(C.byref(desc), *(_ptr(t) for t in (x_new, wk_pk, wv_pk, k_cache, v_cache)),
                                               int(pos), _stream(stream))
    return _check(st, "beagle_xattn_kv_append_prepared", check)


def beagle_xattn_block_kv_append_prepared(desc, params, dw, x_new, k_cache, v_cache, pos, stream=None, *, check=True) -> int:
    st = lib().beagle_xattn_block_kv_append_prepared(
        C.byref(desc), C.byref(params) if params is not None else None, C.byref(dw) if dw is not None else None,
        _ptr(x_new), _ptr(k_cache), _ptr(v_cache), int(pos), _stream(stream))
    return _check(st, "beagle_xattn_block_kv_append_prepared", check)


def beagle_xattn_draft_step_prepared(desc, x_draft, k_cache, v_cache, wq_pk, wo_pk, n_true, tree_mask, mask_words, y, lse,
                                     workspace, stream=None, *, workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_draft_step_prepared(
        C.byref(desc), *(_ptr(t) for t in (x_draft, k_cache, v_cache, wq_pk, wo_pk)), int(n_true), _ptr(tree_mask),
        int(mask_words), _ptr(y), _ptr(lse),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_draft_step_prepared", check)


def beagle_xattn_kv_append(desc, x_new, wk, wv, k_cache, v_cache, pos, workspace, stream=None, *,
                           workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_kv_append(
        C.byref(desc), *(_ptr(t) for t in (x_new, wk, wv, k_cache, v_cache)), int(pos),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_kv_append", check)


def beagle_xattn_workspace_bytes(desc, which) -> int:
    return int(lib().beagle_xattn_workspace_bytes(C.byref(desc), which))


def beagle_xattn_fwd(desc, xq, xkv, wq, wk, wv, wo, y, lse, q_save, k_save, v_save, o_save,
                     workspace=None, stream=None, *, workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_fwd(
        C.byref(desc), *(_ptr(t) for t in (xq, xkv, wq, wk, wv, wo, y, lse, q_save, k_save, v_save, o_save)),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_fwd", check)


def beagle_xattn_bwd(desc, dy, xq, xkv, wq, wk, wv, wo, q_save, k_save, v_save, o_save, lse,
                     dxq, dxkv, dwq, dwk, dwv, dwo, workspace, stream=None, *, workspace_bytes=None,
                     check=True) -> int:
    st = lib().beagle_xattn_bwd(
        C.byref(desc), *(_ptr(t) for t in (dy, xq, xkv, wq, wk, wv, wo, q_save, k_save, v_save, o_save, lse,
                                           dxq, dxkv, dwq, dwk, dwv, dwo)),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_bwd", check)


def beagle_xattn_draft_step(desc, x_draft, k_cache, v_cache, wq, wo, y, lse, workspace, stream=None, *,
                            workspace_bytes=None, check=True) -> int:
    st = lib().beagle_xattn_draft_step(
        C.byref(desc), *(_ptr(t) for t in (x_draft, k_cache, v_cache, wq, wo, y, lse)),
        _ptr(workspace), _nbytes(workspace) if workspace_bytes is None else workspace_bytes, _stream(stream))
    return _check(st, "beagle_xattn_draft_step", check)


BEAGLE_STATIC_SCRATCH_BYTES = 32 << 20
BEAGLE_CLOCK_SLOTS = 2048
BEAGLE_PREPARED_MAX_QUERIES = 16


def beagle_xattn_draft_step_static(desc, x_draft, k_cache, v_cache, wq, wo, y, lse, stream=None, *, check=True) -> int:
    st = lib().beagle_xattn_draft_step_static(
        C.byref(desc), *(_ptr(t) for t in (x_draft, k_cache, v_cache, wq, wo, y, lse)), _stream(stream))
    return _check(st, "beagle_xattn_draft_step_static", check)


def beagle_xattn_mask_row_limit(desc) -> np.ndarray:
    out = np.empty(max(desc.seq_q, 0), np.int32)
    _check(lib().beagle_xattn_mask_row_limit(C.byref(desc), out.ctypes.data), "beagle_xattn_mask_row_limit", True)
    return out


def beagle_xattn_mask_dense(desc) -> np.ndarray:
    out = np.empty((max(desc.seq_q, 0), max(desc.seq_kv, 0)), np.uint8)
    _check(lib().beagle_xattn_mask_dense(C.byref(desc), out.ctypes.data), "beagle_xattn_mask_dense", True)
    return out


def beagle_xattn_tile_map(desc, tq, tk) -> np.ndarray:
    if tq < 1 or tk < 1:
        raise BeagleError(2, "beagle_xattn_tile_map")
    nq, nk = -(-desc.seq_q // tq), -(-desc.seq_kv // tk)
    out = np.empty((max(nq, 0), max(nk, 0)), np.uint8)
    _check(lib().beagle_xattn_tile_map(C.byref(desc), tq, tk, out.ctypes.data), "beagle_xattn_tile_map", True)
    return out


def beagle_xattn_profile_begin() -> None:
    _check(lib().beagle_xattn_profile_begin(), "beagle_xattn_profile_begin", True)


def beagle_xattn_profile_end() -> dict:
    """Returns {kernel name: (launches, total_ms)} for the launches since begin."""
    n = lib().beagle_xattn_profile_end()
    if n < 0:
        raise BeagleError(6, "beagle_xattn_profile_end")
    out = {}
    for i in range(n):
        name, cnt, ms = C.c_char_p(), C.c_int32(), C.c_double()
        _check(lib().beagle_xattn_profile_get(i, C.byref(name), C.byref(cnt), C.byref(ms)),
               "beagle_xattn_profile_get", True)
        out[name.value.decode()] = (cnt.value, ms.value)
    return out


def beagle_xattn_probe_clock(out, stream=None) -> None:
    _check(lib().beagle_xattn_probe_clock(_ptr(out), _stream(stream)), "beagle_xattn_probe_clock", True)


def beagle_xattn_probe_read(buf, nbytes: int, workgroups: int, sink, stream=None) -> None:
    _check(lib().beagle_xattn_probe_read(_ptr(buf), nbytes, workgroups, _ptr(sink), _stream(stream)),
           "beagle_xattn_probe_read", True)


def beagle_xattn_status_string(status: int) -> str:
    return lib().beagle_xattn_status_string(status).decode()


def beagle_xattn_version() -> str:
    return lib().beagle_xattn_version().decode()
