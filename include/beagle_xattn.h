/*
 * beagle_xattn.h -- C ABI of the block-masked cross-attention of Beagle's
 * single-layer draft decoder (paper section 4.1, Eq. 2; training mask of
 * section 4.2; KV-cache decode protocol at the end of section 4.1), for
 * AMD MI355X (gfx950).
 *
 * Notation (0-based; the paper is 1-based)
 *   B batch, S query length, L key length, D model width ("hidden"),
 *   H query heads, G key/value heads (G divides H), d head width,
 *   k window ("block") size, eps window offset in [0, k).
 *   ws(p) = max(0, eps + k * floor((p - eps) / k)) is the start of the window
 *   that holds query p.  Query p may attend key j  iff  j < ws(p).
 *   This is the strict rule "key j is hidden when j >= i" of section 4.1
 *   together with the early-stage rule of section 4.2 that a window hides its
 *   own keys from its own queries; k = 1 is the strict-causal cross mask.
 *   The mask is never materialised on the device (constant space).
 *
 * General conventions
 *   - Every tensor argument is a DEVICE pointer to a contiguous row-major
 *     array (last index fastest), 16-byte aligned, allocated and owned by the
 *     caller.  The library neither allocates, frees nor keeps them.  The two
 *     exceptions are the descriptor (host memory) and the outputs of the
 *     beagle_xattn_mask_* helpers (host memory).
 *   - Element type of activations and weights is desc->io_dtype (float or
 *     bfloat16); sums are always accumulated in float.  lse is always float.
 *   - Weights are stored [in, out] so that Q = Xq * Wq; head h of a projected
 *     tensor occupies columns [h*d, (h+1)*d).  Query head h reads KV head
 *     h / (H / G).
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  Calls return without synchronising.
 *   - Arguments are validated on the host before anything is enqueued: a
 *     status other than BEAGLE_OK / BEAGLE_ERR_HIP means nothing ran.
 *     Nothing throws across this boundary.
 *   - A query with no visible key (ws(p) == 0) gets a zero output row, lse =
 *     -infinity and contributes no gradient.
 *   - Results are run-to-run bitwise reproducible (no floating-point atomics).
 *
 * Rotary position embedding (optional, BEAGLE_FLAG_ROPE)
 *   Section 4.1 leaves positional embeddings out of its equations; the LLaMA /
 *   Vicuna targets rotate queries and keys.  With the flag set, the projected
 *   Q (at the query's sequence position) and K (at the key's) are rotated per
 *   head in the rotate-half convention of those models: channel c < d/2 pairs
 *   with channel c + d/2, angle = position * rope_base^(-2c/d).  V is not
 *   rotated.  q_save / k_save and the decode cache hold the ROTATED rows; the
 *   backward rotates dQ, dK back before the projections' gradients.  In the
 *   simulation step a predicted state stands at its own sequence position.
 *
 * Supported shapes
 *   BEAGLE_F32 : any d <= 128 with d % 4 == 0; D, H*d, G*d multiples of 4.
 *   BEAGLE_BF16: d == 128; D a multiple of 64; every operand smaller than
 *                2 GiB: max(B*S, B*L) * max(D, H*d) * 2 < 2^31 and
 *                D * H*d * 2 < 2^31 (block entry points: the same with F).
 *   B, S, L >= 1 arbitrary (ragged tiles are handled); anything else returns
 *   BEAGLE_ERR_UNSUPPORTED before anything is enqueued -- there is no fallback
 *   path and no slower kernel behind these limits.
 */
#ifndef BEAGLE_XATTN_H
#define BEAGLE_XATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BEAGLE_OK = 0,
  BEAGLE_ERR_NULL = 1,        /* a required pointer is NULL                     */
  BEAGLE_ERR_SHAPE = 2,       /* a size is non-positive or inconsistent         */
  BEAGLE_ERR_UNSUPPORTED = 3, /* valid problem that this build has no kernel for*/
  BEAGLE_ERR_WORKSPACE = 4,   /* workspace missing or smaller than required     */
  BEAGLE_ERR_ALIGN = 5,       /* a device pointer is not 16-byte aligned        */
  BEAGLE_ERR_HIP = 6          /* the HIP runtime reported an error at launch    */
} beagle_status;

typedef enum { BEAGLE_F32 = 0, BEAGLE_BF16 = 1 } beagle_dtype;

enum {
  BEAGLE_FLAG_NEED_DXKV = 1u << 0, /* bwd also produces dxkv                    */
  BEAGLE_FLAG_WGRAD_F32 = 1u << 1, /* bwd writes dwq/dwk/dwv/dwo as float even
                                      when io_dtype is bf16                     */
  BEAGLE_FLAG_ROPE = 1u << 2,      /* rotary position embedding of Q and K, see
                                      rope_base / rope_positions below          */
  BEAGLE_FLAG_STATES_F16 = 1u << 3 /* the key/value source states (xkv; hs of the
                                      block entry points) are stored as IEEE half
                                      precision, as the offline-generated target
                                      states of the paper's training set-up are;
                                      they are converted to io_dtype on the way in
                                      (workspace grows by one [B,L,D] tensor, also
                                      for the forward entry points).  Everything
                                      else, dxkv / dhs included, stays io_dtype.
                                      Training entry points only; D % 8 == 0.    */
};

enum { BEAGLE_WS_FWD = 0, BEAGLE_WS_BWD = 1, BEAGLE_WS_DRAFT = 2, BEAGLE_WS_APPEND = 3, BEAGLE_WS_BWD_SIM = 4,
       BEAGLE_WS_BLOCK_APPEND = 5 };

typedef struct {
  int32_t struct_size;   /* sizeof(beagle_xattn_desc); checked                  */
  int32_t batch;         /* B                                                   */
  int32_t seq_q;         /* S <= 2^30 (draft step: M, the number of draft queries) */
  int32_t seq_kv;        /* L <= 2^30 (training: usually == S)                  */
  int32_t hidden;        /* D                                                   */
  int32_t n_q_heads;     /* H                                                   */
  int32_t n_kv_heads;    /* G, divides H                                        */
  int32_t head_dim;      /* d                                                   */
  int32_t block_size;    /* 1 <= k <= 2^30 (section 4.2 window size)            */
  int32_t block_offset;  /* eps in [0, k) (section 4.2 random offset)           */
  int32_t io_dtype;      /* beagle_dtype                                        */
  float   softmax_scale; /* 0 selects 1/sqrt(d) as in Eq. 2                     */
  uint32_t flags;        /* BEAGLE_FLAG_*; unknown bits are rejected            */
  const int32_t* block_offsets; /* NULL, or DEVICE pointer to B offsets: batch entry
                            b uses eps = block_offsets[b] instead of block_offset
                            (section 4.2's random offset drawn per sequence).
                            Values must lie in [0, k); the kernels reduce them
                            modulo k.  4-byte aligned.  Not used by the draft-step
                            entry points; the host-side beagle_xattn_mask_* /
                            beagle_xattn_tile_map helpers return
                            BEAGLE_ERR_UNSUPPORTED when it is set (inspect one
                            entry at a time through block_offset).              */
  /* Packed batches of sequences of different lengths (training entry points;
   * NULL / 0 for the ordinary [B,S,..] layout; BEAGLE_ERR_UNSUPPORTED for the
   * draft-step entry points).  cu_seqlens_q / cu_seqlens_kv are DEVICE pointers
   * to B + 1 increasing int32 values, first 0, last total_q / total_kv: entry
   * b owns query rows cu_seqlens_q[b] .. cu_seqlens_q[b+1]-1 of the packed
   * [total_q, ..] tensors and key rows likewise.  seq_q / seq_kv are then the
   * LONGEST lengths (every entry holds between 1 and seq_q, seq_kv rows); masks
   * and positions restart in every entry.  Shapes: replace [B,S,..] by
   * [total_q,..] and [B,L,..] by [total_kv,..]; lse (and the workspace's delta)
   * become [H,total_q].  The arrays cannot be checked on the host: offsets
   * that do not describe rows inside the packed tensors are clamped, which
   * gives wrong results but no access outside the buffers.  The simulation
   * entry points need cu_seqlens_q == cu_seqlens_kv.                          */
  const int32_t* cu_seqlens_q;
  const int32_t* cu_seqlens_kv;
  int32_t total_q, total_kv;
  float rope_base;       /* BEAGLE_FLAG_ROPE: frequency base; 0 selects 10000   */
  const int32_t* rope_positions; /* BEAGLE_FLAG_ROPE, decode side only (DEVICE pointer
                            or NULL): draft step -- the sequence positions of its
                            M queries (NULL: all at seq_kv, the position after the
                            cached rows); kv_append -- the positions of the n new
                            rows (NULL: pos + i).  Must be NULL for the training
                            entry points, where position = index.  4-byte aligned. */
} beagle_xattn_desc;

/* Bytes of device workspace that the given entry point needs for `desc`
 * (`which` is BEAGLE_WS_*).  Returns 0 for an invalid descriptor. */
size_t beagle_xattn_workspace_bytes(const beagle_xattn_desc* desc, int which);

/*
 * Forward pass (Eq. 2): Q = Xq Wq, K = Xkv Wk, V = Xkv Wv, masked softmax over
 * the visible keys with scale 1/sqrt(d), O = P V, Y = O Wo.
 *   in : xq [B,S,D], xkv [B,L,D], wq [D,H*d], wk [D,G*d], wv [D,G*d], wo [H*d,D]
 *   out: y [B,S,D]; lse [B,H,S] float, natural-log log-sum-exp of the scaled
 *        visible scores; q_save [B,S,H,d], k_save [B,L,G,d], v_save [B,L,G,d],
 *        o_save [B,S,H,d] in io_dtype -- the tensors the backward pass reuses
 *        (k_save / v_save are also exactly the KV-cache rows of the decode
 *        step).  All eight outputs are required.
 */
beagle_status beagle_xattn_fwd(const beagle_xattn_desc* desc,
    const void* xq, const void* xkv, const void* wq, const void* wk,
    const void* wv, const void* wo,
    void* y, float* lse, void* q_save, void* k_save, void* v_save, void* o_save,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward pass of the same operation (used by the training-time simulation
 * of section 4.2), by recomputing the probabilities from q_save, k_save, lse:
 *   dO = dY Wo^T, dWo = O^T dY, delta = rowsum(dO * O), P = exp(s - lse),
 *   dV = P^T dO, dS = P * (dO V^T - delta), dQ = dS K * scale,
 *   dK = dS^T Q * scale (summed over the H/G query heads of a KV head),
 *   dXq = dQ Wq^T, dWq = Xq^T dQ, dWk = Xkv^T dK, dWv = Xkv^T dV,
 *   dXkv = dK Wk^T + dV Wv^T (only with BEAGLE_FLAG_NEED_DXKV).
 *   in : dy [B,S,D] and the forward's inputs and saved tensors
 *   out: dxq [B,S,D]; dxkv [B,L,D] (NULL allowed unless NEED_DXKV is set);
 *        dwq [D,H*d], dwk, dwv [D,G*d], dwo [H*d,D] in io_dtype, or float with
 *        BEAGLE_FLAG_WGRAD_F32.  Outputs are overwritten, not accumulated.
 */
beagle_status beagle_xattn_bwd(const beagle_xattn_desc* desc,
    const void* dy, const void* xq, const void* xkv, const void* wq,
    const void* wk, const void* wv, const void* wo,
    const void* q_save, const void* k_save, const void* v_save,
    const void* o_save, const float* lse,
    void* dxq, void* dxkv, void* dwq, void* dwk, void* dwv, void* dwo,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Decode-time draft step (section 4.1, KV-cache paragraph): M = desc->seq_q
 * draft query states attend to a cache of L = desc->seq_kv already projected
 * key/value rows; every query sees every cache row (drafted states are not
 * concatenated), so block_size / block_offset are ignored.  desc->batch must
 * be 1.
 *   in : x_draft [M,D], k_cache [L,G,d], v_cache [L,G,d], wq [D,H*d], wo [H*d,D]
 *   out: y [M,D] = softmax(q K^T * scale) V Wo with q = x_draft Wq;
 *        lse [H,M] float.
 */
beagle_status beagle_xattn_draft_step(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache,
    const void* wq, const void* wo, void* y, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * beagle_xattn_draft_step for callers that cannot allocate or hand over device
 * memory of their own for scratch: code under HIP-graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * (bitwise) and kernels as beagle_xattn_draft_step, without the workspace: the
 * partial sums live in a buffer of BEAGLE_STATIC_SCRATCH_BYTES that is part of
 * the library's device image (every GPU the library runs on holds its own copy
 * until the process ends).  The call allocates and frees nothing.
 *   - The first call on a device looks up that device's copy of the buffer
 *     (once; make that call outside graph capture).
 *   - A problem whose beagle_xattn_workspace_bytes(desc, BEAGLE_WS_DRAFT)
 *     exceeds BEAGLE_STATIC_SCRATCH_BYTES returns BEAGLE_ERR_WORKSPACE and
 *     enqueues nothing (the decode configuration of 64 queries, 4096 cache
 *     rows, D = 4096 needs 26 MB).
 *   - All calls on one GPU share the one buffer, whose content is whatever the
 *     last call left (no kernel of the step needs it cleared): calls that may
 *     overlap on one GPU -- different streams, or graphs replayed concurrently
 *     -- race; keep them on one stream.
 */
#define BEAGLE_STATIC_SCRATCH_BYTES (32u << 20)
beagle_status beagle_xattn_draft_step_static(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache,
    const void* wq, const void* wo, void* y, float* lse, void* hip_stream);

/*
 * Late-stage training: one simulated inference step (section 4.2, second
 * half, and the caption of the mask figure).  Keys come from two sources: the
 * true target states xkv under the early-stage mask of beagle_xattn_fwd, and
 * the buffer xpred [B,L,D] of states that the draft model predicted in the
 * earlier simulation steps of this iteration (updated in place between steps
 * with beagle_xattn_sim_save: constant space).  At step sim_step = t >= 0 query p, whose
 * window starts at w0(p) = eps + k*floor((p - eps)/k), also sees predicted key
 * j iff max(w0(p), 0) <= j < min(p, w0(p) + t): the first t positions of its
 * own window that lie before it.  t = 0 is beagle_xattn_fwd; t >= k - 1 shows
 * every earlier position of the window.  Queries are not unrolled (xq is the
 * same in every step); predicted states are projected with the same Wk, Wv.
 * Requires seq_q == seq_kv.
 *   in : as beagle_xattn_fwd, plus xpred [B,L,D]
 *   out: as beagle_xattn_fwd, plus kp_save, vp_save [B,L,G,d] (K, V of xpred)
 */
beagle_status beagle_xattn_fwd_sim(const beagle_xattn_desc* desc,
    const void* xq, const void* xkv, const void* xpred, const void* wq,
    const void* wk, const void* wv, const void* wo, int32_t sim_step,
    void* y, float* lse, void* q_save, void* k_save, void* v_save,
    void* kp_save, void* vp_save, void* o_save,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * In-place update of the predicted-state buffer between two simulated steps
 * (section 4.2, second half: the states predicted at the start of every
 * window are saved after the first step, those of the next position after
 * the second, and so on, always into the same buffer).  After step
 * sim_step = t the row at position t of every window (rows j with
 * j - w0(j) == t, w0 as in beagle_xattn_fwd_sim) takes row j of h; all other
 * rows of xpred keep their content.  h is whatever the caller's draft block
 * produced for every position in step t (the residual adds and the MLP of
 * Eq. 1 are outside this library).  t >= block_size changes nothing.
 *   in    : h [B,L,D] (io dtype, device)
 *   in/out: xpred [B,L,D] (device); h and xpred must not overlap
 * Requires seq_q == seq_kv.  Asynchronous on hip_stream.
 */
beagle_status beagle_xattn_sim_save(const beagle_xattn_desc* desc,
    const void* h, void* xpred, int32_t sim_step, void* hip_stream);

/*
 * Backward of the simulated step: as beagle_xattn_bwd, with the gradient of
 * the predicted-state buffer as an additional output, and with Wk, Wv
 * receiving the contributions of both key sources:
 *   dWk = Xkv^T dK + Xpred^T dKp, dWv likewise, dXpred = dKp Wk^T + dVp Wv^T
 * (rows of xpred that no query sees get exactly zero).
 *   in : as beagle_xattn_bwd, plus xpred, kp_save, vp_save and sim_step
 *   out: as beagle_xattn_bwd, plus dxpred [B,L,D] (required)
 * Workspace: beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD_SIM).
 */
beagle_status beagle_xattn_bwd_sim(const beagle_xattn_desc* desc,
    const void* dy, const void* xq, const void* xkv, const void* xpred,
    const void* wq, const void* wk, const void* wv, const void* wo,
    const void* q_save, const void* k_save, const void* v_save,
    const void* kp_save, const void* vp_save, const void* o_save,
    const float* lse, int32_t sim_step,
    void* dxq, void* dxkv, void* dxpred, void* dwq, void* dwk, void* dwv, void* dwo,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The whole draft block around the attention (section 4.1, Eq. 1):
 *     y = CrossAttn(hs, e) + e          h = MLP(y) + y
 * Eq. 1 fixes the two residual lines and calls the MLP a point-wise
 * feed-forward layer; normalisation and the MLP's form are "layer details"
 * the paper leaves out.  This library takes the layout of the LLaMA / Vicuna
 * targets: every sublayer reads an RMS-normalised copy of its input and each
 * residual adds the un-normalised stream,
 *     xq = RMSNorm(e; g_q)   xkv = RMSNorm(hs; g_kv)   z = RMSNorm(y; g_mlp)
 *     RMSNorm(x; g) = x / sqrt(mean_c(x_c^2) + rms_eps) * g
 *     MLP(z) = (silu(z W_gate) * (z W_up)) W_down,   silu(u) = u / (1 + exp(-u))
 * A NULL gain switches that normalisation off, which is Eq. 1 as printed.
 * The attention inside is exactly beagle_xattn_fwd / beagle_xattn_bwd on (xq, xkv)
 * with desc's mask; the residual adds run in the epilogues of the output
 * projection and of the down projection.
 *
 * All pointers are device pointers (16-byte aligned, caller-owned) except the
 * three structs themselves, which are read on the host during the call.
 */
typedef struct {
  int32_t struct_size;          /* sizeof(beagle_block_params); checked          */
  int32_t ffn;                  /* F, width of the feed-forward layer;
                                   BEAGLE_F32: F % 4 == 0, BEAGLE_BF16: F % 64 == 0 */
  float   rms_eps;              /* >= 0                                          */
  int32_t reserved;             /* 0                                             */
  const void *wq, *wk, *wv, *wo;        /* as beagle_xattn_fwd                   */
  const void *w_gate, *w_up;            /* [D, F]                                */
  const void *w_down;                   /* [F, D]                                */
  const void *g_q, *g_kv, *g_mlp;       /* [D] gains in io_dtype, or NULL        */
} beagle_block_params;

/* Written by beagle_xattn_block_fwd, read by beagle_xattn_block_bwd.  xq_n / r_q, xkv_n /
 * r_kv, z / r_mlp are needed only when the matching gain is given. */
typedef struct {
  void *xq_n;  float *r_q;      /* [B,S,D] normalised e, [B*S] 1/rms             */
  void *xkv_n; float *r_kv;     /* [B,L,D] normalised hs, [B*L]                  */
  void *q, *k, *v, *o; float *lse;      /* as the *_save / lse outputs of beagle_xattn_fwd */
  void *y;                      /* [B,S,D] after the first residual              */
  void *z;     float *r_mlp;    /* [B,S,D] normalised y, [B*S]                   */
  void *u, *w, *m;              /* [B,S,F] z W_gate, z W_up, silu(u) * w         */
  /* simulation entry points only */
  void *xp_n;  float *r_p;      /* [B,L,D] normalised xpred, [B*L] (with g_kv)   */
  void *kp, *vp;                /* [B,L,G,d] K, V of the predicted states        */
} beagle_block_saved;

typedef struct {
  void *de;                     /* [B,S,D]                                       */
  void *dhs;                    /* [B,L,D]; required iff BEAGLE_FLAG_NEED_DXKV   */
  void *dwq, *dwk, *dwv, *dwo;  /* like the weights (io_dtype)                   */
  void *dw_gate, *dw_up, *dw_down;
  float *dg_q, *dg_kv, *dg_mlp; /* [D] float; required iff the gain is given     */
  void *dxpred;                 /* [B,L,D]; simulation entry points only         */
} beagle_block_grads;

enum { BEAGLE_WS_BLOCK_FWD = 0, BEAGLE_WS_BLOCK_BWD = 1, BEAGLE_WS_BLOCK_DRAFT = 2, BEAGLE_WS_BLOCK_BWD_SIM = 3 };

/* Workspace bytes of the two block entry points (`which` is BEAGLE_WS_BLOCK_*);
 * 0 for an invalid descriptor / ffn. */
size_t beagle_xattn_block_workspace_bytes(const beagle_xattn_desc* desc, int32_t ffn, int which);

/*
 * Forward of the block.  in: e [B,S,D], hs [B,L,D]; out: h [B,S,D] and `saved`.
 * BEAGLE_ERR_UNSUPPORTED additionally for D > 12288 when any gain is given and
 * for BEAGLE_FLAG_WGRAD_F32.  Workspace: BEAGLE_WS_BLOCK_FWD (may be 0 bytes).
 */
beagle_status beagle_xattn_block_fwd(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const void* e, const void* hs, void* h, const beagle_block_saved* saved,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of the block: gradients of sum(dh * h) with respect to e, hs
 * (optional), the seven weight matrices and the given gains.
 *   in : dh [B,S,D], e, hs, params, saved (as written by the forward)
 *   out: grads
 * Workspace: BEAGLE_WS_BLOCK_BWD.
 */
beagle_status beagle_xattn_block_bwd(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const void* dh, const void* e, const void* hs, const beagle_block_saved* saved,
    const beagle_block_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The block in a late-stage simulation step (section 4.2, second half): as
 * beagle_xattn_block_fwd / _bwd with the attention of beagle_xattn_fwd_sim /
 * _bwd_sim.  The predicted states xpred [B,L,D] are this block's own earlier
 * outputs h, written into the buffer by beagle_xattn_sim_save; as key/value
 * source states they pass through the same normalisation as hs (g_kv, whose
 * gradient then collects both sources).  sim_step = 0 is the plain block.
 * Requires seq_q == seq_kv.  saved->kp, vp (and xp_n, r_p with g_kv) and
 * grads->dxpred are required.  Workspace: BEAGLE_WS_BLOCK_FWD for the forward,
 * BEAGLE_WS_BLOCK_BWD_SIM for the backward.
 */
beagle_status beagle_xattn_block_fwd_sim(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const void* e, const void* hs, const void* xpred, int32_t sim_step, void* h, const beagle_block_saved* saved,
    void* workspace, size_t workspace_bytes, void* hip_stream);
beagle_status beagle_xattn_block_bwd_sim(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const void* dh, const void* e, const void* hs, const void* xpred, int32_t sim_step,
    const beagle_block_saved* saved, const beagle_block_grads* grads,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The block at decode time (section 4.1, last paragraphs: the same block
 * decodes draft tokens autoregressively against the cached K/V rows): M draft
 * token embeddings through Eq. 1,
 *     y = DraftStep(RMSNorm(x; g_q)) + x        h = MLP(RMSNorm(y; g_mlp)) + y
 * where DraftStep is beagle_xattn_draft_step_tree (n_true = seq_kv and a NULL
 * mask give beagle_xattn_draft_step).  The key/value side (g_kv, wk, wv) is
 * not used here: rows enter the cache through beagle_xattn_kv_append.
 * desc as for the draft step (batch == 1, seq_q = M, seq_kv = cache rows).
 *   in : x_draft [M,D]; k_cache, v_cache [L,G,d]; params (wq, wo, w_gate, w_up,
 *        w_down required; g_q, g_mlp optional); tree mask as in
 *        beagle_xattn_draft_step_tree
 *   out: h [M,D]; lse [H,M] float
 * Workspace: beagle_xattn_block_workspace_bytes(desc, ffn, BEAGLE_WS_BLOCK_DRAFT).
 * BEAGLE_BF16: a handful of rows is HBM-bound on the weights (Wq, Wo and the
 * three feed-forward matrices) and the cache, so every projection is the
 * split-k streaming kernel of the draft step.
 */
beagle_status beagle_xattn_block_draft_step(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const void* x_draft, const void* k_cache, const void* v_cache, int32_t n_true, const uint32_t* tree_mask,
    int32_t mask_words, void* h, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The block's draft step on weights in the decode-time layout (see
 * beagle_xattn_prepare_weights): the two attention projections and the three
 * feed-forward matrices packed, so that each projection is one launch of 16-column strips
 * over the whole of k -- no k split, no partial sums, no launch to add them,
 * and the SiLU gate runs in the epilogue of the gate/up projection.
 *   beagle_xattn_block_prepare_weights: fills the buffers of `dw` (DEVICE,
 *     caller-owned, 16-byte aligned, each the size of its source): wq_pk from
 *     params->wq [D, H*d], wo_pk from params->wo [H*d, D], w_gate_pk, w_up_pk from [D, F], w_down_pk from
 *     [F, D].  Once per model load.  bf16 with D % 128 == 0 and F % 128 == 0,
 *     else BEAGLE_ERR_UNSUPPORTED.  The gains of the two normalisations are
 *     folded into the matrices that read the normalised rows: wq_pk packs
 *     diag(g_q) wq, w_gate_pk and w_up_pk pack diag(g_mlp) w_gate / w_up (each
 *     product rounded to bf16), for whichever of g_q, g_mlp is not NULL.
 *   beagle_xattn_block_draft_step_prepared: beagle_xattn_block_draft_step with
 *     params->wq, wo, w_gate, w_up, w_down replaced by `dw` (those five fields
 *     of params are not read; ffn and rms_eps are, and g_q, g_mlp only as
 *     switches: non-NULL exactly where they were when `dw` was prepared).  The
 *     two normalisations run inside the projections that follow them (the
 *     row factor 1 / sqrt(mean(x^2) + eps) multiplies the finished sums), so
 *     the normalised rows are never rounded to bf16 on their own.  Same definition
 *     of h and lse; sums run in a different fixed order, so results agree with
 *     the plain entry point to rounding, not bitwise.  1 <= seq_q <=
 *     BEAGLE_PREPARED_MAX_QUERIES, bf16, D % 128 == 0, F % 128 == 0;
 *     BEAGLE_ERR_UNSUPPORTED otherwise, before anything is enqueued.
 * Workspace: BEAGLE_WS_BLOCK_DRAFT.
 */
typedef struct {
  int32_t struct_size;          /* sizeof(beagle_block_decode_weights); checked  */
  int32_t reserved;             /* 0                                             */
  void *wq_pk, *wo_pk;          /* packed wq, wo: D * H*d elements each          */
  void *wk_pk, *wv_pk;          /* packed wk, wv: D * G*d elements each; both NULL
                                   if the cache is appended to another way       */
  void *w_gate_pk, *w_up_pk;    /* packed w_gate, w_up: D * F elements each      */
  void *w_down_pk;              /* packed w_down: F * D elements                 */
} beagle_block_decode_weights;
beagle_status beagle_xattn_block_prepare_weights(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const beagle_block_decode_weights* dw, void* hip_stream);
beagle_status beagle_xattn_block_draft_step_prepared(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const beagle_block_decode_weights* dw, const void* x_draft, const void* k_cache, const void* v_cache,
    int32_t n_true, const uint32_t* tree_mask, int32_t mask_words, void* h, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream);
/* beagle_xattn_block_kv_append on dw->wk_pk, dw->wv_pk (which beagle_xattn_block_prepare_weights fills, with
 * diag(g_kv) folded in, when params->wk, wv and both destinations are given): the key/value normalisation and both
 * projections in one launch, no workspace.  Of params only rms_eps is read, and g_kv as a switch.  Up to
 * BEAGLE_PREPARED_MAX_QUERIES new states, bf16, D % 128 == 0; BEAGLE_ERR_UNSUPPORTED otherwise. */
beagle_status beagle_xattn_block_kv_append_prepared(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const beagle_block_decode_weights* dw, const void* x_new, void* k_cache, void* v_cache, int32_t pos,
    void* hip_stream);

/*
 * Cache append for the block: new states (true ones, or drafted ones = earlier
 * outputs h of beagle_xattn_block_draft_step) are key/value source states, so
 * they take the key/value normalisation RMSNorm(.; params->g_kv) before the
 * projections, exactly as hs does in beagle_xattn_block_fwd; then as
 * beagle_xattn_kv_append with params->wk, params->wv (the other fields of params
 * are not read; g_kv NULL gives the plain append).
 * Workspace: beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BLOCK_APPEND).
 */
beagle_status beagle_xattn_block_kv_append(const beagle_xattn_desc* desc, const beagle_block_params* params,
    const void* x_new, void* k_cache, void* v_cache, int32_t pos,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Appending states to the decode cache (section 4.1, KV-cache paragraph: new
 * K_i, V_i are appended as drafting proceeds, and the cache is reset to the
 * true states at the end of a speculative-decoding iteration).  The
 * n = desc->seq_q states x_new (true target states, or drafted states) are
 * projected and written in place,
 *   k_cache[pos + i] = x_new[i] Wk,   v_cache[pos + i] = x_new[i] Wv,   i < n,
 * into a cache with room for desc->seq_kv rows; 0 <= pos, pos + n <= seq_kv.
 * No other row is touched.  Resetting the cache needs no call: the caller
 * stops counting the rows past the true states.  desc->batch must be 1;
 * block_size / block_offset are ignored.
 *   in    : x_new [n,D], wk [D,G*d], wv [D,G*d]
 *   in/out: k_cache, v_cache [seq_kv,G,d]
 * Workspace: beagle_xattn_workspace_bytes(desc, BEAGLE_WS_APPEND) (split-k
 * partial sums of the two projections when n is small).
 */
beagle_status beagle_xattn_kv_append(const beagle_xattn_desc* desc,
    const void* x_new, const void* wk, const void* wv,
    void* k_cache, void* v_cache, int32_t pos,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Draft step with the drafted states concatenated to the cache, under a draft
 * tree (appendix "Ablation Study": the "concate" option with the dynamic
 * drafting tree; tree shape in section 5.1).  The
 * cache holds n_true rows of true states followed by T = desc->seq_kv - n_true
 * rows of drafted states.  Query m sees every true row, and drafted row
 * n_true + t iff bit (t % 32) of tree_mask[m * mask_words + t / 32] is set.
 * 0 <= n_true <= seq_kv; mask_words >= ceil(T / 32); bits at t >= T are
 * ignored; with T == 0 this is beagle_xattn_draft_step and tree_mask may be
 * NULL.  A query that sees no row at all gets y = 0 and lse = -inf.
 *   in : as beagle_xattn_draft_step, plus tree_mask: DEVICE pointer,
 *        uint32 [M, mask_words], 4-byte aligned
 *   out: y [M,D], lse [H,M]
 * Workspace: beagle_xattn_workspace_bytes(desc, BEAGLE_WS_DRAFT).
 */
beagle_status beagle_xattn_draft_step_tree(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache,
    const void* wq, const void* wo, int32_t n_true,
    const uint32_t* tree_mask, int32_t mask_words, void* y, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Decode-time weight layout.  The draft step streams each weight matrix once.
 * Packed for that use, a matrix W [K, N] (row-major, y = a W) is stored as
 * 4 KB blocks of 16 output columns x 128 k, block (m, s) = (k / 128, n / 16) at
 * byte ((m * N/16) + s) * 4096, and inside a block the 16 bytes of piece
 * (j, l), j = 0..3, l = 0..63, at (j * 64 + l) * 16 hold the eight values
 *     W[128 m + 32 j + 8 (l / 16) + e][16 s + l % 16],  e = 0..7
 * -- the order in which the lanes of a wavefront feed them to the matrix
 * instruction.  A workgroup then owns 16 output columns over the whole of k,
 * every load is 1 KB contiguous and the workgroups sweep the matrix front to
 * back together, so the projection needs no k split, no partial sums in memory
 * and no launch to add them.  Weights are fixed while drafting (section 4.1:
 * the draft model is trained beforehand), so packing is paid once per model
 * load, not per step.  A packed matrix has the size of the original.
 *   beagle_xattn_prepare_weights: packs wq [D, H*d], wk, wv [D, G*d] and wo
 *     [H*d, D] into wq_pk, wk_pk, wv_pk, wo_pk (all DEVICE; a source and its
 *     destination may both be NULL to skip that matrix, at least one pair must be
 *     given; a destination must not overlap its source).  bf16 with D % 128 == 0
 *     only (BEAGLE_ERR_UNSUPPORTED otherwise).
 *   beagle_xattn_draft_step_prepared: beagle_xattn_draft_step_tree with wq_pk,
 *     wo_pk in the place of wq, wo (n_true == seq_kv and tree_mask == NULL give
 *     the plain draft step).  Same definition of y and lse; sums run in a
 *     different (fixed) order than in beagle_xattn_draft_step, so results agree
 *     with it to rounding, not bitwise.  Serves 1 <= seq_q <=
 *     BEAGLE_PREPARED_MAX_QUERIES, bf16, D % 128 == 0; BEAGLE_ERR_UNSUPPORTED
 *     otherwise, before anything is enqueued: use the plain entry points there.
 * Workspace: beagle_xattn_workspace_bytes(desc, BEAGLE_WS_DRAFT).
 */
#define BEAGLE_PREPARED_MAX_QUERIES 16
beagle_status beagle_xattn_prepare_weights(const beagle_xattn_desc* desc,
    const void* wq, const void* wk, const void* wv, const void* wo,
    void* wq_pk, void* wk_pk, void* wv_pk, void* wo_pk, void* hip_stream);
/* beagle_xattn_kv_append on packed wk_pk, wv_pk: one launch, no partial sums, hence no workspace.  Serves
 * 1 <= seq_q (the number of new states) <= BEAGLE_PREPARED_MAX_QUERIES, bf16, D % 128 == 0;
 * BEAGLE_ERR_UNSUPPORTED otherwise. */
beagle_status beagle_xattn_kv_append_prepared(const beagle_xattn_desc* desc,
    const void* x_new, const void* wk_pk, const void* wv_pk,
    void* k_cache, void* v_cache, int32_t pos, void* hip_stream);
beagle_status beagle_xattn_draft_step_prepared(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache,
    const void* wq_pk, const void* wo_pk, int32_t n_true,
    const uint32_t* tree_mask, int32_t mask_words, void* y, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- mask / index inspection (HOST memory, integers only, no GPU needed) --
 * These run the same index code that the kernels use, so that it can be
 * compared bit for bit with a mask built independently from the paper. */

/* ws_out[p] = min(ws(p), L) for p in [0,S): the number of keys query p sees. */
beagle_status beagle_xattn_mask_row_limit(const beagle_xattn_desc* desc, int32_t* ws_out);
/* mask_out[p*L + j] = 1 if query p may attend key j, else 0. */
beagle_status beagle_xattn_mask_dense(const beagle_xattn_desc* desc, uint8_t* mask_out);
/* Class of every (query tile, key tile) pair for tiles of tq x tk:
 * cls_out[a * ceil(L/tk) + c] = 0 skip (nothing visible), 1 partial (needs the
 * per-element predicate), 2 full (everything visible).  Section 4.2's block
 * structure is what makes whole-tile skipping possible. */
beagle_status beagle_xattn_tile_map(const beagle_xattn_desc* desc, int32_t tq, int32_t tk, uint8_t* cls_out);

/* ---- per-kernel timing (measurement aid) ---------------------------------
 * Between profile_begin and profile_end every kernel launch of the three
 * entry points is bracketed by HIP events on the launch stream.  profile_end
 * synchronises those events and returns the number of distinct kernel names;
 * profile_get then yields, for index i, the name (static string), the launch
 * count and the summed duration in milliseconds.  Not thread-safe; capacity
 * is 4096 launches per begin/end pair (further launches are not timed). */
beagle_status beagle_xattn_profile_begin(void);
int32_t       beagle_xattn_profile_end(void);
beagle_status beagle_xattn_profile_get(int32_t i, const char** name, int32_t* launches, double* total_ms);

/* ---- streaming-read reference (measurement aid) ----------------------------
 * Enqueues a kernel that does nothing but read `bytes` bytes (a multiple of 16)
 * from the DEVICE buffer `buf` with 16-byte loads, `workgroups` workgroups of
 * 256 threads, eight loads in flight per thread.  Timed by the caller over a
 * buffer it has not touched recently, this is what the memory system delivers
 * to a read-only kernel: the practical ceiling next to which the decode step's
 * achieved bandwidth (section 4.1, KV-cache paragraph: the step streams the
 * cache once) is reported.  `sink` is a DEVICE pointer to 4 writable bytes
 * (written only if the XOR of all words read equals one magic value).        */
beagle_status beagle_xattn_probe_read(const void* buf, size_t bytes, int32_t workgroups, void* sink, void* hip_stream);

/* ---- clock sample (measurement aid) -----------------------------------------
 * Enqueues a kernel of 1024 one-wave workgroups, each of which writes two
 * 64-bit counters, read back to back, into the slot of the compute unit it ran
 * on: out[2 s] = that unit's shader-cycle counter, out[2 s + 1] = the device's
 * constant-rate clock (100 MHz); s = 0 .. BEAGLE_CLOCK_SLOTS - 1 is formed from
 * the XCD number and the unit's position bits.  `out` is a DEVICE buffer of
 * BEAGLE_CLOCK_SLOTS x 16 writable bytes, 8-byte aligned, zeroed by the caller
 * before its first use; a slot whose unit ran no workgroup keeps its old
 * contents.  Cycle counters of different units are not aligned: take
 * differences within one slot only.  Two samples on one stream around a region
 * of work give (delta cycles) / (delta clock) x 100 MHz = the mean shader clock
 * over that region; the benchmark's timed loops report it next to their
 * throughput, since the matrix-pipe peak that the throughput is set against
 * assumes 2.4 GHz.  Not part of the method.                                    */
#define BEAGLE_CLOCK_SLOTS 2048
beagle_status beagle_xattn_probe_clock(void* out, void* hip_stream);

const char* beagle_xattn_status_string(beagle_status s);
/* "major.minor" of this ABI. */
const char* beagle_xattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BEAGLE_XATTN_H */
