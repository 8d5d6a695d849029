// C-ABI entry points: argument validation, workspace carving, and the order in
// which the kernels of the hot path are enqueued.  No arithmetic lives here.
#include "../../include/beagle_xattn.h"
#include "common.h"
#include "api_internal.h"

#include <math.h>
#include <mutex>
#include <string.h>

using namespace beagle;

namespace beagle {
namespace detail {

constexpr uint32_t KNOWN_FLAGS = BEAGLE_FLAG_NEED_DXKV | BEAGLE_FLAG_WGRAD_F32 | BEAGLE_FLAG_ROPE | BEAGLE_FLAG_STATES_F16;
beagle_status check_desc(const beagle_xattn_desc* c, bool draft, Dims* out) {
  if (!c) return BEAGLE_ERR_NULL;
  if (c->struct_size != (int32_t)sizeof(beagle_xattn_desc)) return BEAGLE_ERR_SHAPE;
  if (c->batch < 1 || c->seq_q < 1 || c->seq_kv < 1 || c->hidden < 1 || c->n_q_heads < 1 ||
      c->n_kv_heads < 1 || c->head_dim < 1)
    return BEAGLE_ERR_SHAPE;
  if (c->n_q_heads % c->n_kv_heads) return BEAGLE_ERR_SHAPE;
  if (!draft && (c->block_size < 1 || c->block_offset < 0 || c->block_offset >= c->block_size))
    return BEAGLE_ERR_SHAPE;
  if (draft && c->batch != 1) return BEAGLE_ERR_SHAPE;
  // the index code works in int32: lengths and window sizes up to 2^30 keep every intermediate in range
  if (c->seq_q > (1 << 30) || c->seq_kv > (1 << 30) || (!draft && c->block_size > (1 << 30))) return BEAGLE_ERR_UNSUPPORTED;
  if (c->flags & ~KNOWN_FLAGS) return BEAGLE_ERR_UNSUPPORTED;
  if (c->io_dtype != BEAGLE_F32 && c->io_dtype != BEAGLE_BF16) return BEAGLE_ERR_UNSUPPORTED;
  if (!(c->softmax_scale >= 0.f) || isinf(c->softmax_scale)) return BEAGLE_ERR_SHAPE;
  Dims d;
  d.B = c->batch; d.S = c->seq_q; d.L = c->seq_kv; d.D = c->hidden;
  d.H = c->n_q_heads; d.G = c->n_kv_heads; d.d = c->head_dim;
  d.HD = d.H * d.d; d.GD = d.G * d.d;
  d.bf16 = c->io_dtype == BEAGLE_BF16;
  d.esz = d.bf16 ? 2 : 4;
  // grid dimensions and 32-bit row counts used by the kernels
  if (d.B > 65535 || d.H > 65535) return BEAGLE_ERR_UNSUPPORTED;
  if (d.B * d.S > INT32_MAX / 2 || d.B * d.L > INT32_MAX / 2 || d.HD > INT32_MAX / 2 || d.D > INT32_MAX / 2)
    return BEAGLE_ERR_UNSUPPORTED;
  if (d.bf16) {
    if (d.d != 128 || d.D % 64) return BEAGLE_ERR_UNSUPPORTED;
    // the bf16 kernels address one batch entry's Q / K / V slab, and the decode step a whole weight matrix,
    // through 32-bit buffer descriptors
    const int64_t lim = (int64_t)1 << 31;
    if (d.S * d.HD * 2 >= lim || d.L * d.GD * 2 >= lim) return BEAGLE_ERR_UNSUPPORTED;
    // ... and the projection kernels every operand as a whole: activations [rows, D], projected rows
    // [rows, H*d], weights [D, H*d].  There is no slower kernel behind these limits.
    const int64_t rows = c->cu_seqlens_q ? (int64_t)(c->total_q > c->total_kv ? c->total_q : c->total_kv)
                                         : d.B * (d.S > d.L ? d.S : d.L);
    const int64_t width = d.D > d.HD ? d.D : d.HD;
    if (rows * width * 2 >= lim || d.D * d.HD * 2 >= lim) return BEAGLE_ERR_UNSUPPORTED;
  } else {
    if (d.d > 128 || d.d % 4 || d.D % 4) return BEAGLE_ERR_UNSUPPORTED;
  }
  d.scale = c->softmax_scale > 0.f ? c->softmax_scale : (float)(1.0 / sqrt((double)d.d));
  d.mask.k = draft ? 1 : c->block_size;
  d.mask.eps = draft ? 0 : c->block_offset;
  d.mask.seq_kv = (int32_t)d.L;
  d.mask.all_visible = draft ? 1 : 0;
  if (c->block_offsets && (((uintptr_t)c->block_offsets) & 3u)) return BEAGLE_ERR_ALIGN;
  d.eps_b = draft ? nullptr : c->block_offsets;
  d.Tq = d.B * d.S; d.Tk = d.B * d.L; d.cu_q = d.cu_kv = nullptr;
  if (c->cu_seqlens_q || c->cu_seqlens_kv) {
    if (draft) return BEAGLE_ERR_UNSUPPORTED;
    if (!c->cu_seqlens_q || !c->cu_seqlens_kv) return BEAGLE_ERR_NULL;
    if ((((uintptr_t)c->cu_seqlens_q) | ((uintptr_t)c->cu_seqlens_kv)) & 3u) return BEAGLE_ERR_ALIGN;
    // every entry holds between 1 and S (L) rows
    if (c->total_q < d.B || c->total_q > d.B * d.S || c->total_kv < d.B || c->total_kv > d.B * d.L) return BEAGLE_ERR_SHAPE;
    d.Tq = c->total_q; d.Tk = c->total_kv; d.cu_q = c->cu_seqlens_q; d.cu_kv = c->cu_seqlens_kv;
  }
  d.kv_f16 = (c->flags & BEAGLE_FLAG_STATES_F16) != 0;
  if (d.kv_f16 && (draft || d.D % 8)) return BEAGLE_ERR_UNSUPPORTED;
  d.rope = (c->flags & BEAGLE_FLAG_ROPE) != 0;
  d.rope_base = 10000.f; d.rope_pos = nullptr;
  if (d.rope) {
    if (!(c->rope_base >= 0.f) || isinf(c->rope_base)) return BEAGLE_ERR_SHAPE;
    if (c->rope_base > 0.f) d.rope_base = c->rope_base;
    if (d.d % 4) return BEAGLE_ERR_UNSUPPORTED;
    if (c->rope_positions) {
      if (!draft) return BEAGLE_ERR_UNSUPPORTED;           // training: position = index
      if (((uintptr_t)c->rope_positions) & 3u) return BEAGLE_ERR_ALIGN;
      d.rope_pos = c->rope_positions;
    }
  }
  *out = d;
  return BEAGLE_OK;
}

BwdWs bwd_layout(const Dims& d) {
  BwdWs w; size_t o = 0;
  w.dO = o; o += align_up((size_t)(d.Tq * d.HD) * d.esz);
  w.dQ = o; o += align_up((size_t)(d.Tq * d.HD) * d.esz);
  w.dK = o; o += align_up((size_t)(d.Tk * d.GD) * d.esz);
  w.dV = o; o += align_up((size_t)(d.Tk * d.GD) * d.esz);
  w.delta = o; o += align_up((size_t)(d.B * d.H * d.S) * sizeof(float));
  w.dwpart = o; if (split_kv_wgrad(d)) o += align_up((size_t)(4 * d.D * d.GD) * sizeof(float));
  w.attn = o;
  w.total = o;
  return w;
}

// The three weight gradients dWq, dWk, dWv are one grouped launch of 256 x 256 tiles.  Under grouped-query attention dWk
// and dWv are narrow, and the launch can end in a round of tiles that fills a fraction of the 256 compute units (H 32 /
// G 8 at D 4096: 256 + 64 + 64 tiles, i.e. a full round and a half-empty one of the same length).  Then dWq goes alone
// and dWk, dWv go as four problems of half the depth each (the first and the second half of the key/value rows, float
// results), followed by one pass that adds the halves: a full round, a full round of half the length, and a sum that
// moves 10 bytes per element.  Chosen by counting rounds, with the sum priced at a tenth of an 8192-row round per 128
// tiles (measured: 84 MB in about 20 us against 190 us); the result is a fixed function of the shapes.
bool split_kv_wgrad(const Dims& d) {
  if (!d.bf16 || d.Tk < 128) return false;
  auto tiles = [](int64_t m, int64_t n) { return ((m + 255) / 256) * ((n + 255) / 256); };
  const int64_t tq = tiles(d.D, d.HD), tkv = tiles(d.D, d.GD);
  if (tq + 2 * tkv < 256 || 4 * d.D * d.GD * (int64_t)sizeof(float) >= ((int64_t)1 << 31)) return false;
  auto rounds = [](int64_t t) { return (double)((t + 255) / 256); };
  const double together = rounds(tq + 2 * tkv);
  const double apart = rounds(tq) + 0.5 * rounds(4 * tkv) + 0.1 * (2.0 * (double)tkv / 128.0) * (8192.0 / (double)d.Tk);
  return apart < 0.9 * together;
}

AttnArgs attn_args(const Dims& d) {
  AttnArgs a; memset(&a, 0, sizeof(a));
  a.B = (int32_t)d.B; a.S = (int32_t)d.S; a.L = (int32_t)d.L; a.H = (int32_t)d.H; a.G = (int32_t)d.G;
  a.d = (int32_t)d.d; a.scale = d.scale; a.mask = d.mask; a.eps_b = d.eps_b;
  a.cu_q = d.cu_q; a.cu_kv = d.cu_kv; a.Tq = (int32_t)d.Tq; a.Tk = (int32_t)d.Tk;
  return a;
}

// C[M,N] = A[M,K] * B  with B stored [K,N] (weights [in,out])
GemmArgs gemm_nn(const void* A, const void* W, void* C, int64_t M, int64_t N, int64_t K) {
  GemmArgs g; memset(&g, 0, sizeof(g));
  g.A = A; g.B = W; g.C = C; g.M = (int32_t)M; g.N = (int32_t)N; g.K = (int32_t)K;
  g.lda = K; g.ldb = N; g.ldc = N; g.a_kmajor = 1; g.b_kmajor = 0;
  return g;
}
// C[M,N] = A[M,K] * W^T  with W stored [N,K]
GemmArgs gemm_nt(const void* A, const void* W, void* C, int64_t M, int64_t N, int64_t K) {
  GemmArgs g = gemm_nn(A, W, C, M, N, K);
  g.ldb = K; g.b_kmajor = 1;
  return g;
}
// C[M,N] = X^T * Y  with X stored [K,M], Y stored [K,N]
GemmArgs gemm_tn(const void* X, const void* Y, void* C, int64_t M, int64_t N, int64_t K, bool c_f32) {
  GemmArgs g = gemm_nn(X, Y, C, M, N, K);
  g.lda = M; g.a_kmajor = 0; g.c_is_f32 = c_f32 ? 1 : 0;
  return g;
}

GemmGroup group1(const GemmArgs& a) { GemmGroup g; memset(&g, 0, sizeof(g)); g.count = 1; g.p[0] = a; return g; }

void run_gemm(const Dims& d, const GemmGroup& g, hipStream_t s, const char* name) {
  if (d.bf16) launch_gemm_bf16(g, s, name); else launch_gemm_f32(g, s, name);
}

beagle_status hip_status() { return hipGetLastError() == hipSuccess ? BEAGLE_OK : BEAGLE_ERR_HIP; }

// Half-precision key/value source states: bytes of the converted copy (kept at the END of every workspace), and
// the conversion itself.  `need` is the entry point's whole workspace requirement.
size_t states_ws(const Dims& d) { return d.kv_f16 ? align_up((size_t)(d.Tk * d.D) * d.esz) : 0; }
const void* states_in(const Dims& d, const void* xkv, void* workspace, size_t need, hipStream_t s) {
  if (!d.kv_f16) return xkv;
  void* dst = (char*)workspace + need - states_ws(d);
  launch_cvt_f16(d.bf16, xkv, dst, d.Tk * d.D, s);
  return dst;
}

RopeArgs rope_args(const Dims& d, bool inverse) {
  RopeArgs r; memset(&r, 0, sizeof(r));
  r.nb = (int32_t)d.B;
  r.d = (int32_t)d.d; r.base = d.rope_base; r.inverse = inverse ? 1 : 0;
  return r;
}
void rope_add(RopeArgs& r, void* x, int64_t rows, int64_t period, int64_t heads, int32_t pos0, const int32_t* pos,
              const int32_t* cu) {
  const int i = r.n++;
  r.cu[i] = cu;
  r.x[i] = x; r.rows[i] = rows; r.period[i] = (int32_t)period; r.heads[i] = (int32_t)heads; r.pos0[i] = pos0; r.pos[i] = pos;
}

// Projections, masked attention, output projection (+ y_res in its epilogue if given).
void xattn_fwd_run(const Dims& d, const void* xq, const void* xkv, const void* wq, const void* wk, const void* wv,
                   const void* wo, void* y, float* lse, void* q_save, void* k_save, void* v_save, void* o_save,
                   const void* y_res, hipStream_t s) {
  GemmGroup qkv; memset(&qkv, 0, sizeof(qkv));
  qkv.count = 3;
  qkv.p[0] = gemm_nn(xq, wq, q_save, d.Tq, d.HD, d.D);
  qkv.p[1] = gemm_nn(xkv, wk, k_save, d.Tk, d.GD, d.D);
  qkv.p[2] = gemm_nn(xkv, wv, v_save, d.Tk, d.GD, d.D);
  run_gemm(d, qkv, s, "proj_qkv");
  if (d.rope) {
    RopeArgs r = rope_args(d, false);
    rope_add(r, q_save, d.Tq, d.S, d.H, 0, nullptr, d.cu_q);
    rope_add(r, k_save, d.Tk, d.L, d.G, 0, nullptr, d.cu_kv);
    launch_rope(d.bf16, r, s, "rope_qk");
  }

  AttnArgs a = attn_args(d);
  a.q = q_save; a.k = k_save; a.v = v_save; a.o = o_save; a.lse = lse;
  if (d.bf16) launch_attn_fwd_bf16(a, s); else launch_attn_fwd_f32(a, s);

  GemmArgs out = gemm_nn(o_save, wo, y, d.Tq, d.D, d.HD);
  out.R = y_res; out.ldr = d.D;
  run_gemm(d, group1(out), s, "proj_out");
}

// All gradients of the attention op; `base` is a workspace of BEAGLE_WS_BWD bytes.  dxq_res, if given, is added
// to dxq in the epilogue of its GEMM.
void xattn_bwd_run(const Dims& d, bool need_dxkv, bool wf32, const void* dy, const void* xq, const void* xkv,
                   const void* wq, const void* wk, const void* wv, const void* wo, const void* q_save,
                   const void* k_save, const void* v_save, const void* o_save, const float* lse, void* dxq,
                   void* dxkv, void* dwq, void* dwk, void* dwv, void* dwo, char* base, const void* dxq_res,
                   hipStream_t s) {
  const BwdWs w = bwd_layout(d);
  void* dO = base + w.dO; void* dQ = base + w.dQ; void* dK = base + w.dK; void* dV = base + w.dV;
  float* delta = (float*)(base + w.delta);
  const int64_t Mq = d.Tq, Mk = d.Tk;

  // dO = dY Wo^T ; dWo = O^T dY
  run_gemm(d, group1(gemm_nt(dy, wo, dO, Mq, d.HD, d.D)), s, "bwd_dout");
  run_gemm(d, group1(gemm_tn(o_save, dy, dwo, d.HD, d.D, Mq, wf32)), s, "bwd_dwo");

  AttnArgs a = attn_args(d);
  a.q = q_save; a.k = k_save; a.v = v_save; a.o = (void*)o_save; a.lse = (float*)lse;
  a.dout = dO; a.dq = dQ; a.dk = dK; a.dv = dV; a.delta = delta;
  if (d.bf16) launch_attn_bwd_bf16(a, base + w.attn, s); else launch_attn_bwd_f32(a, s);
  if (d.rope) {   // dQ, dK are gradients of the rotated rows: rotate them back
    RopeArgs r = rope_args(d, true);
    rope_add(r, dQ, Mq, d.S, d.H, 0, nullptr, d.cu_q);
    rope_add(r, dK, Mk, d.L, d.G, 0, nullptr, d.cu_kv);
    launch_rope(d.bf16, r, s, "bwd_rope_qk");
  }

  // input gradients
  {
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 1;
    g.p[0] = gemm_nt(dQ, wq, dxq, Mq, d.D, d.HD);
    g.p[0].R = dxq_res; g.p[0].ldr = d.D;
    if (need_dxkv) {
      // deeper problem first: dXkv contracts over the K and the V columns
      g.count = 2;
      g.p[1] = g.p[0];
      g.p[0] = gemm_nt(dK, wk, dxkv, Mk, d.D, d.GD);
      g.p[0].A2 = dV; g.p[0].B2 = wv; g.p[0].K2 = (int32_t)d.GD; g.p[0].lda2 = d.GD; g.p[0].ldb2 = d.GD;
    }
    run_gemm(d, g, s, "bwd_dx");
  }
  // weight gradients
  if (split_kv_wgrad(d)) {
    run_gemm(d, group1(gemm_tn(xq, dQ, dwq, d.D, d.HD, Mq, wf32)), s, "bwd_dwq");
    const int64_t kh = (Mk / 2) & ~(int64_t)63, pe = d.D * d.GD;      // rows of the first half; elements of a partial
    float* part = (float*)(base + w.dwpart);
    const char* xh = (const char*)xkv + (size_t)(kh * d.D) * d.esz;
    const char* dKh = (const char*)dK + (size_t)(kh * d.GD) * d.esz;
    const char* dVh = (const char*)dV + (size_t)(kh * d.GD) * d.esz;
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 4;
    g.p[0] = gemm_tn(xh, dKh, part + pe, d.D, d.GD, Mk - kh, true);   // the deeper halves first
    g.p[1] = gemm_tn(xh, dVh, part + 3 * pe, d.D, d.GD, Mk - kh, true);
    g.p[2] = gemm_tn(xkv, dK, part, d.D, d.GD, kh, true);
    g.p[3] = gemm_tn(xkv, dV, part + 2 * pe, d.D, d.GD, kh, true);
    run_gemm(d, g, s, "bwd_dwkv");
    SumPairArgs sp;
    sp.count = 2;
    sp.a[0] = part; sp.b[0] = part + pe; sp.out[0] = dwk;
    sp.a[1] = part + 2 * pe; sp.b[1] = part + 3 * pe; sp.out[1] = dwv;
    launch_sum_pairs(sp, pe, wf32, s, "bwd_dwkv_sum");
  } else {
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 3;
    g.p[0] = gemm_tn(xq, dQ, dwq, d.D, d.HD, Mq, wf32);
    g.p[1] = gemm_tn(xkv, dK, dwk, d.D, d.GD, Mk, wf32);
    g.p[2] = gemm_tn(xkv, dV, dwv, d.D, d.GD, Mk, wf32);
    run_gemm(d, g, s, "bwd_dw");
  }
}

// The simulation step's forward: as xattn_fwd_run, plus the predicted states' K / V and the band merge.
void xattn_fwd_sim_run(const Dims& d, const void* xq, const void* xkv, const void* xpred, const void* wq, const void* wk,
                       const void* wv, const void* wo, int32_t sim_step, void* y, float* lse, void* q_save, void* k_save,
                       void* v_save, void* kp_save, void* vp_save, void* o_save, const void* y_res, hipStream_t s) {
  GemmGroup qkv; memset(&qkv, 0, sizeof(qkv));
  qkv.count = 3;
  qkv.p[0] = gemm_nn(xq, wq, q_save, d.Tq, d.HD, d.D);
  qkv.p[1] = gemm_nn(xkv, wk, k_save, d.Tk, d.GD, d.D);
  qkv.p[2] = gemm_nn(xkv, wv, v_save, d.Tk, d.GD, d.D);
  run_gemm(d, qkv, s, "proj_qkv");
  GemmGroup kvp; memset(&kvp, 0, sizeof(kvp));
  kvp.count = 2;
  kvp.p[0] = gemm_nn(xpred, wk, kp_save, d.Tk, d.GD, d.D);
  kvp.p[1] = gemm_nn(xpred, wv, vp_save, d.Tk, d.GD, d.D);
  run_gemm(d, kvp, s, "proj_kvp");
  if (d.rope) {   // a predicted state stands at its own sequence position
    RopeArgs r = rope_args(d, false);
    rope_add(r, q_save, d.Tq, d.S, d.H, 0, nullptr, d.cu_q);
    rope_add(r, k_save, d.Tk, d.L, d.G, 0, nullptr, d.cu_kv);
    rope_add(r, kp_save, d.Tk, d.L, d.G, 0, nullptr, d.cu_kv);
    launch_rope(d.bf16, r, s, "rope_qk");
  }

  SimArgs sa; memset(&sa, 0, sizeof(sa));
  sa.a = attn_args(d);
  sa.a.q = q_save; sa.a.k = k_save; sa.a.v = v_save; sa.a.o = o_save; sa.a.lse = lse;
  sa.kp = kp_save; sa.vp = vp_save; sa.t = sim_step; sa.is_bf16 = d.bf16 ? 1 : 0;
  if (d.bf16) launch_attn_fwd_bf16(sa.a, s); else launch_attn_fwd_f32(sa.a, s);
  if (sim_step > 0) launch_sim_band_fwd(sa, s);

  GemmArgs out = gemm_nn(o_save, wo, y, d.Tq, d.D, d.HD);
  out.R = y_res; out.ldr = d.D;
  run_gemm(d, group1(out), s, "proj_out");
}

// The simulation step's backward; `base` is a workspace of BEAGLE_WS_BWD_SIM bytes (without the converted states).
void xattn_bwd_sim_run(const Dims& d, bool need_dxkv, bool wf32, const void* dy, const void* xq, const void* xkv,
                       const void* xpred, const void* wq, const void* wk, const void* wv, const void* wo,
                       const void* q_save, const void* k_save, const void* v_save, const void* kp_save,
                       const void* vp_save, const void* o_save, const float* lse, int32_t sim_step, void* dxq, void* dxkv,
                       void* dxpred, void* dwq, void* dwk, void* dwv, void* dwo, char* base, const void* dxq_res,
                       hipStream_t s) {
  const BwdWs w = bwd_layout(d);
  void* dO = base + w.dO; void* dQ = base + w.dQ; void* dK = base + w.dK; void* dV = base + w.dV;
  float* delta = (float*)(base + w.delta);
  size_t extra = 0;
  if (d.bf16) { AttnArgs t = attn_args(d); extra = attn_bwd_bf16_ws_bytes(t); }
  const size_t kvb = align_up((size_t)(d.Tk * d.GD) * d.esz);
  void* dKp = base + w.total + align_up(extra);
  void* dVp = (char*)dKp + kvb;
  const int64_t Mq = d.Tq, Mk = d.Tk;

  run_gemm(d, group1(gemm_nt(dy, wo, dO, Mq, d.HD, d.D)), s, "bwd_dout");
  run_gemm(d, group1(gemm_tn(o_save, dy, dwo, d.HD, d.D, Mq, wf32)), s, "bwd_dwo");

  // true-key part: the main kernels, given the merged LSE and delta = rowsum(dO * O) of the merged O
  SimArgs sa; memset(&sa, 0, sizeof(sa));
  sa.a = attn_args(d);
  sa.a.q = q_save; sa.a.k = k_save; sa.a.v = v_save; sa.a.o = (void*)o_save; sa.a.lse = (float*)lse;
  sa.a.dout = dO; sa.a.dq = dQ; sa.a.dk = dK; sa.a.dv = dV; sa.a.delta = delta;
  sa.kp = kp_save; sa.vp = vp_save; sa.dkp = dKp; sa.dvp = dVp; sa.t = sim_step; sa.is_bf16 = d.bf16 ? 1 : 0;
  if (d.bf16) launch_attn_bwd_bf16(sa.a, base + w.attn, s); else launch_attn_bwd_f32(sa.a, s);
  // predicted-key band: adds to dQ, writes dKp and dVp (zeros where nothing is seen)
  launch_sim_band_bwd(sa, s);
  if (d.rope) {
    RopeArgs r = rope_args(d, true);
    rope_add(r, dQ, Mq, d.S, d.H, 0, nullptr, d.cu_q);
    rope_add(r, dK, Mk, d.L, d.G, 0, nullptr, d.cu_kv);
    rope_add(r, dKp, Mk, d.L, d.G, 0, nullptr, d.cu_kv);
    launch_rope(d.bf16, r, s, "bwd_rope_qk");
  }

  {
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 2;
    g.p[0] = gemm_nt(dKp, wk, dxpred, Mk, d.D, d.GD);
    g.p[0].A2 = dVp; g.p[0].B2 = wv; g.p[0].K2 = (int32_t)d.GD; g.p[0].lda2 = d.GD; g.p[0].ldb2 = d.GD;
    g.p[1] = gemm_nt(dQ, wq, dxq, Mq, d.D, d.HD);
    g.p[1].R = dxq_res; g.p[1].ldr = d.D;
    if (need_dxkv) {
      g.count = 3;
      g.p[2] = g.p[1];
      g.p[1] = gemm_nt(dK, wk, dxkv, Mk, d.D, d.GD);
      g.p[1].A2 = dV; g.p[1].B2 = wv; g.p[1].K2 = (int32_t)d.GD; g.p[1].lda2 = d.GD; g.p[1].ldb2 = d.GD;
    }
    run_gemm(d, g, s, "bwd_dx");
  }
  {
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 3;
    g.p[0] = gemm_tn(xkv, dK, dwk, d.D, d.GD, Mk, wf32);        // two k segments: true and predicted rows
    g.p[0].A2 = xpred; g.p[0].B2 = dKp; g.p[0].K2 = (int32_t)Mk; g.p[0].lda2 = d.D; g.p[0].ldb2 = d.GD;
    g.p[1] = gemm_tn(xkv, dV, dwv, d.D, d.GD, Mk, wf32);
    g.p[1].A2 = xpred; g.p[1].B2 = dVp; g.p[1].K2 = (int32_t)Mk; g.p[1].lda2 = d.D; g.p[1].ldb2 = d.GD;
    g.p[2] = gemm_tn(xq, dQ, dwq, d.D, d.HD, Mq, wf32);
    run_gemm(d, g, s, "bwd_dw");
  }
}

// K / V rows of the n = d.S new states into cache rows pos .. pos + n - 1 (+ rotary embedding of the K rows).
void kv_append_run(const Dims& d, const void* x_new, const void* wk, const void* wv, void* k_cache, void* v_cache,
                   int32_t pos, void* workspace, hipStream_t s, float packed_norm_eps) {
  // rows pos .. pos + n - 1 of the caches are the output matrices (leading dimension G*d)
  char* kdst = (char*)k_cache + (size_t)pos * d.GD * d.esz;
  char* vdst = (char*)v_cache + (size_t)pos * d.GD * d.esz;
  if (packed_norm_eps == packed_norm_eps) {      // not NaN: packed weights (the caller has checked strip_gemm_fits)
    launch_kv_append_strip_bf16(x_new, wk, wv, kdst, vdst, (int32_t)d.S, (int32_t)d.GD, (int32_t)d.D, packed_norm_eps, s);
  } else if (d.bf16 && kv_append_bf16_fits((int32_t)d.S, (int32_t)d.GD, (int32_t)d.D)) {
    // a handful of states: HBM-bound on Wk and Wv, so the split-k streaming projection of the draft step
    launch_kv_append_bf16(x_new, wk, wv, kdst, vdst, (int32_t)d.S, (int32_t)d.GD, (int32_t)d.D, workspace, s);
  } else {
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 2;
    g.p[0] = gemm_nn(x_new, wk, kdst, d.S, d.GD, d.D);
    g.p[1] = gemm_nn(x_new, wv, vdst, d.S, d.GD, d.D);
    run_gemm(d, g, s, "kv_append");
  }
  if (d.rope) {   // the new K rows at their sequence positions (given, or the row indices)
    RopeArgs r = rope_args(d, false);
    rope_add(r, kdst, d.S, d.S, d.G, pos, d.rope_pos);
    launch_rope(d.bf16, r, s, "kv_append_rope");
  }
}

}  // namespace detail
}  // namespace beagle
using namespace beagle::detail;

// ------------------------------------------------------------------ profiler
namespace beagle {
namespace {
constexpr int PROF_CAP = 4096;
struct ProfState {
  bool on = false;
  int n = 0;
  hipEvent_t ev0[PROF_CAP], ev1[PROF_CAP];
  const char* name[PROF_CAP];
  int have_events = 0;
  // aggregated results
  int n_names = 0;
  const char* agg_name[64];
  int agg_count[64];
  double agg_ms[64];
} g_prof;
}  // namespace

void prof_before(const char* name, hipStream_t s) {
  if (!g_prof.on || g_prof.n >= g_prof.have_events) return;
  g_prof.name[g_prof.n] = name;
  (void)hipEventRecord(g_prof.ev0[g_prof.n], s);
}
void prof_after(hipStream_t s) {
  if (!g_prof.on || g_prof.n >= g_prof.have_events) return;
  (void)hipEventRecord(g_prof.ev1[g_prof.n], s);
  ++g_prof.n;
}
}  // namespace beagle

extern "C" {

beagle_status beagle_xattn_profile_begin(void) {
  while (g_prof.have_events < PROF_CAP) {
    int i = g_prof.have_events;
    if (hipEventCreate(&g_prof.ev0[i]) != hipSuccess) return BEAGLE_ERR_HIP;
    if (hipEventCreate(&g_prof.ev1[i]) != hipSuccess) { (void)hipEventDestroy(g_prof.ev0[i]); return BEAGLE_ERR_HIP; }
    ++g_prof.have_events;
  }
  g_prof.n = 0; g_prof.n_names = 0; g_prof.on = true;
  return BEAGLE_OK;
}

int32_t beagle_xattn_profile_end(void) {
  g_prof.on = false;
  g_prof.n_names = 0;
  for (int i = 0; i < g_prof.n; ++i) {
    if (hipEventSynchronize(g_prof.ev1[i]) != hipSuccess) return -1;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.ev0[i], g_prof.ev1[i]) != hipSuccess) return -1;
    int k = 0;
    for (; k < g_prof.n_names; ++k) if (!strcmp(g_prof.agg_name[k], g_prof.name[i])) break;
    if (k == g_prof.n_names) {
      if (k == 64) continue;
      g_prof.agg_name[k] = g_prof.name[i]; g_prof.agg_count[k] = 0; g_prof.agg_ms[k] = 0.0; ++g_prof.n_names;
    }
    g_prof.agg_count[k] += 1; g_prof.agg_ms[k] += ms;
  }
  g_prof.n = 0;
  return g_prof.n_names;
}

beagle_status beagle_xattn_profile_get(int32_t i, const char** name, int32_t* launches, double* total_ms) {
  if (!name || !launches || !total_ms) return BEAGLE_ERR_NULL;
  if (i < 0 || i >= g_prof.n_names) return BEAGLE_ERR_SHAPE;
  *name = g_prof.agg_name[i]; *launches = g_prof.agg_count[i]; *total_ms = g_prof.agg_ms[i];
  return BEAGLE_OK;
}

const char* beagle_xattn_status_string(beagle_status s) {
  switch (s) {
    case BEAGLE_OK: return "ok";
    case BEAGLE_ERR_NULL: return "required pointer is NULL";
    case BEAGLE_ERR_SHAPE: return "invalid or inconsistent size";
    case BEAGLE_ERR_UNSUPPORTED: return "unsupported configuration";
    case BEAGLE_ERR_WORKSPACE: return "workspace missing or too small";
    case BEAGLE_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case BEAGLE_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

beagle_status beagle_xattn_probe_read(const void* buf, size_t bytes, int32_t workgroups, void* sink, void* hip_stream) {
  if (!buf || !sink) return BEAGLE_ERR_NULL;
  if (!aligned16(buf) || (((uintptr_t)sink) & 3u)) return BEAGLE_ERR_ALIGN;
  if (bytes < 16 || workgroups < 1 || workgroups > 65535) return BEAGLE_ERR_SHAPE;
  (void)hipGetLastError();
  launch_read_probe(buf, (int64_t)bytes, workgroups, (uint32_t*)sink, (hipStream_t)hip_stream);
  return hip_status();
}

beagle_status beagle_xattn_probe_clock(void* out, void* hip_stream) {
  if (!out) return BEAGLE_ERR_NULL;
  if (((uintptr_t)out) & 7u) return BEAGLE_ERR_ALIGN;
  (void)hipGetLastError();
  launch_clock_probe((uint64_t*)out, (hipStream_t)hip_stream);
  return hip_status();
}

const char* beagle_xattn_version(void) { return "1.0"; }

// ------------------------------------------------------------- mask helpers
beagle_status beagle_xattn_mask_row_limit(const beagle_xattn_desc* desc, int32_t* ws_out) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  if (d.eps_b) return BEAGLE_ERR_UNSUPPORTED;   // per-entry offsets live on the device: inspect one entry at a time
  if (!ws_out) return BEAGLE_ERR_NULL;
  for (int32_t p = 0; p < d.S; ++p) ws_out[p] = row_limit(p, d.mask);
  return BEAGLE_OK;
}

beagle_status beagle_xattn_mask_dense(const beagle_xattn_desc* desc, uint8_t* mask_out) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  if (d.eps_b) return BEAGLE_ERR_UNSUPPORTED;   // per-entry offsets live on the device: inspect one entry at a time
  if (!mask_out) return BEAGLE_ERR_NULL;
  for (int64_t p = 0; p < d.S; ++p) {
    int32_t lim = row_limit((int32_t)p, d.mask);
    for (int64_t j = 0; j < d.L; ++j) mask_out[p * d.L + j] = j < lim ? 1 : 0;
  }
  return BEAGLE_OK;
}

beagle_status beagle_xattn_tile_map(const beagle_xattn_desc* desc, int32_t tq, int32_t tk, uint8_t* cls_out) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  if (d.eps_b) return BEAGLE_ERR_UNSUPPORTED;   // per-entry offsets live on the device: inspect one entry at a time
  if (!cls_out) return BEAGLE_ERR_NULL;
  if (tq < 1 || tk < 1) return BEAGLE_ERR_SHAPE;
  const int64_t nq = (d.S + tq - 1) / tq, nk = (d.L + tk - 1) / tk;
  for (int64_t a = 0; a < nq; ++a)
    for (int64_t c = 0; c < nk; ++c) {
      int32_t q0 = (int32_t)(a * tq), q1 = (int32_t)((a + 1) * tq < d.S ? (a + 1) * tq : d.S);
      int32_t j0 = (int32_t)(c * tk), j1 = (int32_t)((c + 1) * tk < d.L ? (c + 1) * tk : d.L);
      cls_out[a * nk + c] = (uint8_t)tile_class(q0, q1, j0, j1, d.mask);
    }
  return BEAGLE_OK;
}

// ---------------------------------------------------------------- workspace
size_t beagle_xattn_workspace_bytes(const beagle_xattn_desc* desc, int which) {
  Dims d;
  if (check_desc(desc, which == BEAGLE_WS_DRAFT || which == BEAGLE_WS_APPEND || which == BEAGLE_WS_BLOCK_APPEND, &d) != BEAGLE_OK)
    return 0;
  switch (which) {
    case BEAGLE_WS_FWD: return WS_ALIGN + states_ws(d);   // nothing beyond the saved tensors (and the converted states)
    case BEAGLE_WS_BWD: {
      BwdWs w = bwd_layout(d);
      size_t extra = 0;
      if (d.bf16) { AttnArgs a = attn_args(d); extra = attn_bwd_bf16_ws_bytes(a); }
      return w.total + align_up(extra) + states_ws(d);
    }
    case BEAGLE_WS_DRAFT:
      if (d.bf16) return align_up(decode_bf16_ws_bytes((int32_t)d.S, (int32_t)d.L, (int32_t)d.H, (int32_t)d.d, (int32_t)d.D));
      return align_up((size_t)(2 * d.S * d.HD) * d.esz);
    case BEAGLE_WS_BWD_SIM: {
      BwdWs w = bwd_layout(d);
      size_t extra = 0;
      if (d.bf16) { AttnArgs a = attn_args(d); extra = attn_bwd_bf16_ws_bytes(a); }
      return w.total + align_up(extra) + 2 * align_up((size_t)(d.Tk * d.GD) * d.esz) + states_ws(d);   // + dKp, dVp
    }
    case BEAGLE_WS_APPEND:
    case BEAGLE_WS_BLOCK_APPEND: {
      size_t n = WS_ALIGN;
      if (d.bf16 && kv_append_bf16_fits((int32_t)d.S, (int32_t)d.GD, (int32_t)d.D))
        n += align_up(kv_append_bf16_ws_bytes((int32_t)d.S, (int32_t)d.GD, (int32_t)d.D));
      if (which == BEAGLE_WS_BLOCK_APPEND)   // + the normalised states and their 1/rms
        n += align_up((size_t)(d.S * d.D) * d.esz) + align_up((size_t)d.S * sizeof(float));
      return n;
    }
    default: return 0;
  }
}

// ------------------------------------------------------------------ forward
beagle_status beagle_xattn_fwd(const beagle_xattn_desc* desc,
    const void* xq, const void* xkv, const void* wq, const void* wk, const void* wv, const void* wo,
    void* y, float* lse, void* q_save, void* k_save, void* v_save, void* o_save,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  const void* ptrs[] = {xq, xkv, wq, wk, wv, wo, y, lse, q_save, k_save, v_save, o_save};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  const size_t need_ws = beagle_xattn_workspace_bytes(desc, BEAGLE_WS_FWD);
  if (d.kv_f16) {
    if (!workspace) return BEAGLE_ERR_NULL;
    if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
    if (workspace_bytes < need_ws) return BEAGLE_ERR_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();

  xkv = states_in(d, xkv, workspace, need_ws, s);
  xattn_fwd_run(d, xq, xkv, wq, wk, wv, wo, y, lse, q_save, k_save, v_save, o_save, nullptr, s);
  return hip_status();
}

// ----------------------------------------------------------------- backward
beagle_status beagle_xattn_bwd(const beagle_xattn_desc* desc,
    const void* dy, const void* xq, const void* xkv, const void* wq, const void* wk, const void* wv,
    const void* wo, const void* q_save, const void* k_save, const void* v_save, const void* o_save,
    const float* lse, void* dxq, void* dxkv, void* dwq, void* dwk, void* dwv, void* dwo,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  const bool need_dxkv = desc->flags & BEAGLE_FLAG_NEED_DXKV;
  const void* ptrs[] = {dy, xq, xkv, wq, wk, wv, wo, q_save, k_save, v_save, o_save, lse,
                        dxq, dwq, dwk, dwv, dwo, workspace};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  if (need_dxkv && !dxkv) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  if (dxkv && !aligned16(dxkv)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  if (workspace_bytes < beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD)) return BEAGLE_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();

  xkv = states_in(d, xkv, workspace, beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD), s);
  xattn_bwd_run(d, need_dxkv, d.bf16 && (desc->flags & BEAGLE_FLAG_WGRAD_F32), dy, xq, xkv, wq, wk, wv, wo, q_save, k_save,
                v_save, o_save, lse, dxq, dxkv, dwq, dwk, dwv, dwo, (char*)workspace, nullptr, s);
  return hip_status();
}

// ----------------------------------------------- late-stage simulation step
beagle_status beagle_xattn_fwd_sim(const beagle_xattn_desc* desc,
    const void* xq, const void* xkv, const void* xpred, const void* wq, const void* wk, const void* wv,
    const void* wo, int32_t sim_step, void* y, float* lse, void* q_save, void* k_save, void* v_save,
    void* kp_save, void* vp_save, void* o_save, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  const void* ptrs[] = {xq, xkv, xpred, wq, wk, wv, wo, y, lse, q_save, k_save, v_save, kp_save, vp_save, o_save};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  if (sim_step < 0 || d.S != d.L || d.Tq != d.Tk) return BEAGLE_ERR_SHAPE;
  const size_t need_ws = beagle_xattn_workspace_bytes(desc, BEAGLE_WS_FWD);
  if (d.kv_f16) {
    if (!workspace) return BEAGLE_ERR_NULL;
    if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
    if (workspace_bytes < need_ws) return BEAGLE_ERR_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  xkv = states_in(d, xkv, workspace, need_ws, s);

  xattn_fwd_sim_run(d, xq, xkv, xpred, wq, wk, wv, wo, sim_step, y, lse, q_save, k_save, v_save, kp_save, vp_save, o_save,
                    nullptr, s);
  return hip_status();
}

beagle_status beagle_xattn_sim_save(const beagle_xattn_desc* desc, const void* h, void* xpred, int32_t sim_step,
                                    void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  if (!h || !xpred) return BEAGLE_ERR_NULL;
  if (!aligned16(h) || !aligned16(xpred)) return BEAGLE_ERR_ALIGN;
  if (sim_step < 0 || d.S != d.L || d.Tq != d.Tk) return BEAGLE_ERR_SHAPE;
  if ((d.D * (int64_t)d.esz) % 16) return BEAGLE_ERR_UNSUPPORTED;
  if (sim_step >= desc->block_size) return BEAGLE_OK;      // every window is already full
  (void)hipGetLastError();
  launch_sim_save(h, xpred, (int)d.B, (int)d.L, d.D * (int64_t)d.esz, desc->block_size, desc->block_offset, d.eps_b, sim_step,
                  d.cu_q, (int)d.Tq, (hipStream_t)hip_stream);
  return hip_status();
}

beagle_status beagle_xattn_bwd_sim(const beagle_xattn_desc* desc,
    const void* dy, const void* xq, const void* xkv, const void* xpred, const void* wq, const void* wk,
    const void* wv, const void* wo, const void* q_save, const void* k_save, const void* v_save,
    const void* kp_save, const void* vp_save, const void* o_save, const float* lse, int32_t sim_step,
    void* dxq, void* dxkv, void* dxpred, void* dwq, void* dwk, void* dwv, void* dwo,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, false, &d);
  if (st != BEAGLE_OK) return st;
  const bool need_dxkv = desc->flags & BEAGLE_FLAG_NEED_DXKV;
  const void* ptrs[] = {dy, xq, xkv, xpred, wq, wk, wv, wo, q_save, k_save, v_save, kp_save, vp_save, o_save, lse,
                        dxq, dxpred, dwq, dwk, dwv, dwo, workspace};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  if (need_dxkv && !dxkv) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  if (dxkv && !aligned16(dxkv)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  if (workspace_bytes < beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD_SIM)) return BEAGLE_ERR_WORKSPACE;
  if (sim_step < 0 || d.S != d.L || d.Tq != d.Tk) return BEAGLE_ERR_SHAPE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  xkv = states_in(d, xkv, workspace, beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD_SIM), s);

  xattn_bwd_sim_run(d, need_dxkv, d.bf16 && (desc->flags & BEAGLE_FLAG_WGRAD_F32), dy, xq, xkv, xpred, wq, wk, wv, wo, q_save,
                    k_save, v_save, kp_save, vp_save, o_save, lse, sim_step, dxq, dxkv, dxpred, dwq, dwk, dwv, dwo,
                    (char*)workspace, nullptr, s);
  return hip_status();
}

// --------------------------------------------------------------- draft step
namespace {
// shared by the plain and the draft-tree decode entry points
beagle_status draft_step_impl(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache, const void* wq, const void* wo,
    int32_t n_true, const uint32_t* tree, int32_t words,
    void* y, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream, bool wo_packed = false) {   // wo_packed: wq and wo are both packed
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  if (wo_packed && !(d.bf16 && strip_gemm_fits((int32_t)d.S, (int32_t)d.D, (int32_t)d.HD) &&
                     strip_gemm_fits((int32_t)d.S, (int32_t)d.HD, (int32_t)d.D))) return BEAGLE_ERR_UNSUPPORTED;
  const void* ptrs[] = {x_draft, k_cache, v_cache, wq, wo, y, lse, workspace};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  if (workspace_bytes < beagle_xattn_workspace_bytes(desc, BEAGLE_WS_DRAFT)) return BEAGLE_ERR_WORKSPACE;
  if (n_true < 0 || n_true > d.L) return BEAGLE_ERR_SHAPE;
  const int64_t T = d.L - n_true;
  if (T > 0) {
    if (!tree) return BEAGLE_ERR_NULL;
    if (((uintptr_t)tree) % 4) return BEAGLE_ERR_ALIGN;
    if (words < (T + 31) / 32) return BEAGLE_ERR_SHAPE;
  } else {
    tree = nullptr; words = 0;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();

  if (d.bf16) {
    DecodeArgs a; memset(&a, 0, sizeof(a));
    a.M = (int32_t)d.S; a.L = (int32_t)d.L; a.H = (int32_t)d.H; a.G = (int32_t)d.G; a.d = (int32_t)d.d;
    a.D = (int32_t)d.D; a.scale = d.scale;
    a.x = x_draft; a.kc = k_cache; a.vc = v_cache; a.y = y; a.lse = lse; a.ws = workspace;
    if (wo_packed) { a.wq_pk = wq; a.wo_pk = wo; a.x_norm_eps = -1.f; } else { a.wq = wq; a.wo = wo; }
    a.tree = tree; a.n_true = n_true; a.tree_words = words;
    a.rope = d.rope ? 1 : 0; a.rope_base = d.rope_base; a.rope_pos = d.rope_pos;
    launch_decode_bf16(a, s);
    return hip_status();
  }
  char* base = (char*)workspace;
  void* q = base;
  void* o = base + (size_t)(d.S * d.HD) * d.esz;
  launch_gemm_f32(group1(gemm_nn(x_draft, wq, q, d.S, d.HD, d.D)), s, "draft_proj_q");
  if (d.rope) {   // the M queries at their own positions, or all at the position after the cached rows
    RopeArgs r = rope_args(d, false);
    rope_add(r, q, d.S, d.rope_pos ? d.S : 1, d.H, (int32_t)d.L, d.rope_pos);
    launch_rope(false, r, s, "draft_rope_q");
  }
  AttnArgs a = attn_args(d);
  a.q = q; a.k = k_cache; a.v = v_cache; a.o = o; a.lse = lse;
  a.tree = tree; a.n_true = n_true; a.tree_words = words;
  launch_attn_fwd_f32(a, s);
  launch_gemm_f32(group1(gemm_nn(o, wo, y, d.S, d.D, d.HD)), s, "draft_proj_out");
  return hip_status();
}
}  // namespace

beagle_status beagle_xattn_draft_step(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache, const void* wq, const void* wo,
    void* y, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int32_t L = desc ? desc->seq_kv : 0;
  return draft_step_impl(desc, x_draft, k_cache, v_cache, wq, wo, L, nullptr, 0, y, lse, workspace, workspace_bytes,
                         hip_stream);
}

// The draft step without a caller-provided workspace: the scratch buffer is part of the device image.
// In host code `scratch` is only a handle for hipGetSymbolAddress; kernels get the address it resolves to.
namespace {
static __device__ __align__(256) unsigned char scratch[BEAGLE_STATIC_SCRATCH_BYTES];
constexpr int SCRATCH_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_addr[SCRATCH_MAX_DEVICES];      // per device: every GPU holds its own copy at its own address
beagle_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SCRATCH_MAX_DEVICES) return BEAGLE_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return BEAGLE_ERR_HIP; }
    g_scratch_addr[dev] = p;
  }
  *out = g_scratch_addr[dev];
  return BEAGLE_OK;
}
}  // namespace

beagle_status beagle_xattn_draft_step_static(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache, const void* wq, const void* wo,
    void* y, float* lse, void* hip_stream) {
  const size_t need = beagle_xattn_workspace_bytes(desc, BEAGLE_WS_DRAFT);   // 0: the descriptor check below says why
  if (need > BEAGLE_STATIC_SCRATCH_BYTES) return BEAGLE_ERR_WORKSPACE;
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != BEAGLE_OK) return st;
  return draft_step_impl(desc, x_draft, k_cache, v_cache, wq, wo, desc->seq_kv, nullptr, 0, y, lse, ws,
                         BEAGLE_STATIC_SCRATCH_BYTES, hip_stream);
}

beagle_status beagle_xattn_draft_step_tree(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache, const void* wq, const void* wo,
    int32_t n_true, const uint32_t* tree_mask, int32_t mask_words, void* y, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  return draft_step_impl(desc, x_draft, k_cache, v_cache, wq, wo, n_true, tree_mask, mask_words, y, lse, workspace,
                         workspace_bytes, hip_stream);
}

beagle_status beagle_xattn_prepare_weights(const beagle_xattn_desc* desc,
    const void* wq, const void* wk, const void* wv, const void* wo,
    void* wq_pk, void* wk_pk, void* wv_pk, void* wo_pk, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  const void* src[] = {wq, wk, wv, wo};
  void* dst[] = {wq_pk, wk_pk, wv_pk, wo_pk};
  int given = 0;
  for (int i = 0; i < 4; ++i) {
    if ((!src[i]) != (!dst[i])) return BEAGLE_ERR_NULL;
    if (src[i]) ++given;
  }
  if (!given) return BEAGLE_ERR_NULL;
  for (int i = 0; i < 4; ++i) if (src[i] && (!aligned16(src[i]) || !aligned16(dst[i]))) return BEAGLE_ERR_ALIGN;
  if (!d.bf16 || d.D % 128 || d.HD % 128 || d.GD % 16) return BEAGLE_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  if (wq) launch_pack_strips_bf16(wq, wq_pk, (int32_t)d.D, (int32_t)d.HD, nullptr, s);
  if (wk) launch_pack_strips_bf16(wk, wk_pk, (int32_t)d.D, (int32_t)d.GD, nullptr, s);
  if (wv) launch_pack_strips_bf16(wv, wv_pk, (int32_t)d.D, (int32_t)d.GD, nullptr, s);
  if (wo) launch_pack_strips_bf16(wo, wo_pk, (int32_t)d.HD, (int32_t)d.D, nullptr, s);
  return hip_status();
}

beagle_status beagle_xattn_kv_append_prepared(const beagle_xattn_desc* desc,
    const void* x_new, const void* wk_pk, const void* wv_pk, void* k_cache, void* v_cache, int32_t pos, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  const void* ptrs[] = {x_new, wk_pk, wv_pk, k_cache, v_cache};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  if (!(d.bf16 && strip_gemm_fits((int32_t)d.S, (int32_t)d.GD, (int32_t)d.D))) return BEAGLE_ERR_UNSUPPORTED;
  if (pos < 0 || (int64_t)pos + d.S > d.L) return BEAGLE_ERR_SHAPE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  kv_append_run(d, x_new, wk_pk, wv_pk, k_cache, v_cache, pos, nullptr, s, -1.f);
  return hip_status();
}

beagle_status beagle_xattn_draft_step_prepared(const beagle_xattn_desc* desc,
    const void* x_draft, const void* k_cache, const void* v_cache, const void* wq_pk, const void* wo_pk,
    int32_t n_true, const uint32_t* tree_mask, int32_t mask_words, void* y, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  return draft_step_impl(desc, x_draft, k_cache, v_cache, wq_pk, wo_pk, n_true, tree_mask, mask_words, y, lse, workspace,
                         workspace_bytes, hip_stream, true);
}

beagle_status beagle_xattn_kv_append(const beagle_xattn_desc* desc,
    const void* x_new, const void* wk, const void* wv, void* k_cache, void* v_cache, int32_t pos,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  const void* ptrs[] = {x_new, wk, wv, k_cache, v_cache, workspace};
  for (const void* p : ptrs) if (!p) return BEAGLE_ERR_NULL;
  for (const void* p : ptrs) if (!aligned16(p)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  if (workspace_bytes < beagle_xattn_workspace_bytes(desc, BEAGLE_WS_APPEND)) return BEAGLE_ERR_WORKSPACE;
  if (pos < 0 || (int64_t)pos + d.S > d.L) return BEAGLE_ERR_SHAPE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  kv_append_run(d, x_new, wk, wv, k_cache, v_cache, pos, workspace, s);
  return hip_status();
}

}  // extern "C"

