// C-ABI entry points of the draft block around the attention (section 4.1, Eq. 1): training forward / backward,
// the late-stage simulation variants, the decode-time step and the cache append.  Validation, workspace carving
// and launch order only; the attention inside is the same host code as the plain entry points.
#include "api_internal.h"

#include <math.h>
#include <string.h>

using namespace beagle;
using namespace beagle::detail;

// ------------------------------------------- the draft block around the attention (Eq. 1)
namespace beagle {
namespace {

struct BlockWs { size_t dm, dw, dz, dy, dxq, dxkv, part, attn, total; };

BlockWs block_bwd_layout(const Dims& d, int64_t F) {
  BlockWs w; size_t o = 0;
  const size_t Mq = (size_t)(d.Tq), Mk = (size_t)(d.Tk);
  w.dm = o; o += align_up(Mq * F * d.esz);          // dm, then du in place
  w.dw = o; o += align_up(Mq * F * d.esz);
  w.dz = o; o += align_up(Mq * d.D * d.esz);
  w.dy = o; o += align_up(Mq * d.D * d.esz);
  w.dxq = o; o += align_up(Mq * d.D * d.esz);
  w.dxkv = o; o += align_up(Mk * d.D * d.esz);
  w.part = o; o += align_up((size_t)RMS_BWD_MAX_PARTS * d.D * sizeof(float));
  w.attn = o;
  w.total = o;
  return w;
}

beagle_status check_block(const beagle_xattn_desc* desc, const beagle_block_params* p, Dims* d, bool draft = false) {
  beagle_status st = check_desc(desc, draft, d);
  if (st != BEAGLE_OK) return st;
  if (!p) return BEAGLE_ERR_NULL;
  if (p->struct_size != (int32_t)sizeof(beagle_block_params) || p->ffn < 1 || p->reserved != 0) return BEAGLE_ERR_SHAPE;
  if (!(p->rms_eps >= 0.f) || isinf(p->rms_eps)) return BEAGLE_ERR_SHAPE;
  if (p->ffn % (d->bf16 ? 64 : 4)) return BEAGLE_ERR_UNSUPPORTED;
  if (desc->flags & BEAGLE_FLAG_WGRAD_F32) return BEAGLE_ERR_UNSUPPORTED;
  if ((p->g_q || p->g_kv || p->g_mlp) && d->D > RMS_MAX_D) return BEAGLE_ERR_UNSUPPORTED;
  if (d->B * d->S * (int64_t)p->ffn > (int64_t)INT32_MAX * 64) return BEAGLE_ERR_UNSUPPORTED;
  // bf16: the feed-forward operands [rows, F], [D, F] through 32-bit buffer descriptors, like the attention's
  if (d->bf16 && ((d->Tq > d->D ? d->Tq : d->D) * (int64_t)p->ffn * 2 >= ((int64_t)1 << 31))) return BEAGLE_ERR_UNSUPPORTED;
  return BEAGLE_OK;
}

}  // namespace
}  // namespace beagle

namespace beagle {
namespace {
// decode-time block: xn [M,D], 1/rms [M], y [M,D], z [M,D], then the draft step's and the feed-forward's own space
struct BlockDraftWs { size_t xn, rinv, y, z, u, w, m, step, mlp, total; };
BlockDraftWs block_draft_layout(const beagle_xattn_desc* desc, const Dims& d, int64_t F) {
  BlockDraftWs w; size_t o = 0;
  const size_t MD = align_up((size_t)(d.S * d.D) * d.esz), MF = align_up((size_t)(d.S * F) * d.esz);
  w.xn = o; o += MD;
  w.rinv = o; o += align_up((size_t)d.S * sizeof(float));
  w.y = o; o += MD;
  w.z = o; o += MD;
  w.u = o; o += d.bf16 ? 0 : MF;             // fp32 path: gate / up projections and their product in full
  w.w = o; o += d.bf16 ? 0 : MF;
  w.m = o; o += d.bf16 ? 0 : MF;
  w.step = o; o += beagle_xattn_workspace_bytes(desc, BEAGLE_WS_DRAFT);
  w.mlp = o; o += d.bf16 ? align_up(block_mlp_bf16_ws_bytes((int32_t)d.S, (int32_t)d.D, (int32_t)F)) : 0;
  w.total = o;
  return w;
}
}  // namespace
}  // namespace beagle

size_t beagle_xattn_block_workspace_bytes(const beagle_xattn_desc* desc, int32_t ffn, int which) {
  Dims d;
  if (which == BEAGLE_WS_BLOCK_DRAFT) {
    if (check_desc(desc, true, &d) != BEAGLE_OK || ffn < 1 || ffn % (d.bf16 ? 64 : 4)) return 0;
    return block_draft_layout(desc, d, ffn).total;
  }
  if (check_desc(desc, false, &d) != BEAGLE_OK || ffn < 1 || ffn % (d.bf16 ? 64 : 4)) return 0;
  if (which == BEAGLE_WS_BLOCK_FWD) return WS_ALIGN + states_ws(d);
  if (which == BEAGLE_WS_BLOCK_BWD)
    return block_bwd_layout(d, ffn).total + beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD);
  if (which == BEAGLE_WS_BLOCK_BWD_SIM)   // + the gradient of the normalised predicted states
    return block_bwd_layout(d, ffn).total + align_up((size_t)(d.Tk * d.D) * d.esz) +
           beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BWD_SIM);
  return 0;
}

namespace {
// sim: the attention is the simulation step's (xpred, sim_step); otherwise the early-stage one
beagle_status block_fwd_impl(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* e, const void* hs, bool sim, const void* xpred, int32_t sim_step, void* h, const beagle_block_saved* sv,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_block(desc, p, &d);
  if (st != BEAGLE_OK) return st;
  if (!sv) return BEAGLE_ERR_NULL;
  if (sim) {
    if (!xpred || !sv->kp || !sv->vp || (p->g_kv && (!sv->xp_n || !sv->r_p))) return BEAGLE_ERR_NULL;
    const void* more[] = {xpred, sv->kp, sv->vp, sv->xp_n, sv->r_p};
    for (const void* q : more) if (q && !aligned16(q)) return BEAGLE_ERR_ALIGN;
    if (sim_step < 0 || d.S != d.L || d.Tq != d.Tk) return BEAGLE_ERR_SHAPE;
  }
  const void* req[] = {e, hs, h, p->wq, p->wk, p->wv, p->wo, p->w_gate, p->w_up, p->w_down,
                       sv->q, sv->k, sv->v, sv->o, sv->lse, sv->y, sv->u, sv->w, sv->m};
  for (const void* q : req) if (!q) return BEAGLE_ERR_NULL;
  if (p->g_q && (!sv->xq_n || !sv->r_q)) return BEAGLE_ERR_NULL;
  if (p->g_kv && (!sv->xkv_n || !sv->r_kv)) return BEAGLE_ERR_NULL;
  if (p->g_mlp && (!sv->z || !sv->r_mlp)) return BEAGLE_ERR_NULL;
  const void* all[] = {e, hs, h, p->wq, p->wk, p->wv, p->wo, p->w_gate, p->w_up, p->w_down, p->g_q, p->g_kv, p->g_mlp,
                       sv->xq_n, sv->r_q, sv->xkv_n, sv->r_kv, sv->q, sv->k, sv->v, sv->o, sv->lse, sv->y, sv->z,
                       sv->r_mlp, sv->u, sv->w, sv->m};
  for (const void* q : all) if (q && !aligned16(q)) return BEAGLE_ERR_ALIGN;
  const size_t need_ws = beagle_xattn_block_workspace_bytes(desc, p->ffn, BEAGLE_WS_BLOCK_FWD);
  if (d.kv_f16) {
    if (!workspace) return BEAGLE_ERR_NULL;
    if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
    if (workspace_bytes < need_ws) return BEAGLE_ERR_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const int64_t Mq = d.Tq, Mk = d.Tk, F = p->ffn;
  const int D = (int)d.D;
  hs = states_in(d, hs, workspace, need_ws, s);

  const void* xq = e; const void* xkv = hs;
  if (p->g_q) { launch_rmsnorm_fwd(d.bf16, e, p->g_q, sv->xq_n, sv->r_q, Mq, D, p->rms_eps, s, "norm_q"); xq = sv->xq_n; }
  if (p->g_kv) { launch_rmsnorm_fwd(d.bf16, hs, p->g_kv, sv->xkv_n, sv->r_kv, Mk, D, p->rms_eps, s, "norm_kv"); xkv = sv->xkv_n; }
  // y = CrossAttn(xkv, xq) + e: the residual is the epilogue operand of the output projection
  if (sim) {
    const void* xp = xpred;     // predicted states are key/value source states: same normalisation as hs
    if (p->g_kv) { launch_rmsnorm_fwd(d.bf16, xpred, p->g_kv, sv->xp_n, sv->r_p, Mk, D, p->rms_eps, s, "norm_pred"); xp = sv->xp_n; }
    xattn_fwd_sim_run(d, xq, xkv, xp, p->wq, p->wk, p->wv, p->wo, sim_step, sv->y, sv->lse, sv->q, sv->k, sv->v, sv->kp,
                      sv->vp, sv->o, e, s);
  } else {
    xattn_fwd_run(d, xq, xkv, p->wq, p->wk, p->wv, p->wo, sv->y, sv->lse, sv->q, sv->k, sv->v, sv->o, e, s);
  }
  const void* z = sv->y;
  if (p->g_mlp) { launch_rmsnorm_fwd(d.bf16, sv->y, p->g_mlp, sv->z, sv->r_mlp, Mq, D, p->rms_eps, s, "norm_mlp"); z = sv->z; }
  GemmGroup gu; memset(&gu, 0, sizeof(gu));
  gu.count = 2;
  gu.p[0] = gemm_nn(z, p->w_gate, sv->u, Mq, F, d.D);
  gu.p[1] = gemm_nn(z, p->w_up, sv->w, Mq, F, d.D);
  run_gemm(d, gu, s, "mlp_gate_up");
  launch_silu_mul_fwd(d.bf16, sv->u, sv->w, sv->m, Mq * F, s);
  // h = m W_down + y
  GemmArgs dn = gemm_nn(sv->m, p->w_down, h, Mq, d.D, F);
  dn.R = sv->y; dn.ldr = d.D;
  run_gemm(d, group1(dn), s, "mlp_down");
  return hip_status();
}

beagle_status block_bwd_impl(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* dh, const void* e, const void* hs, bool sim, const void* xpred, int32_t sim_step,
    const beagle_block_saved* sv, const beagle_block_grads* gr, void* workspace, size_t workspace_bytes,
    void* hip_stream) {
  Dims d; beagle_status st = check_block(desc, p, &d);
  if (st != BEAGLE_OK) return st;
  if (!sv || !gr) return BEAGLE_ERR_NULL;
  if (sim) {
    if (!xpred || !sv->kp || !sv->vp || !gr->dxpred || (p->g_kv && (!sv->xp_n || !sv->r_p))) return BEAGLE_ERR_NULL;
    const void* more[] = {xpred, sv->kp, sv->vp, sv->xp_n, sv->r_p, gr->dxpred};
    for (const void* q : more) if (q && !aligned16(q)) return BEAGLE_ERR_ALIGN;
    if (sim_step < 0 || d.S != d.L || d.Tq != d.Tk) return BEAGLE_ERR_SHAPE;
  }
  const int ws_kind = sim ? BEAGLE_WS_BLOCK_BWD_SIM : BEAGLE_WS_BLOCK_BWD;
  const bool need_dhs = desc->flags & BEAGLE_FLAG_NEED_DXKV;
  const void* req[] = {dh, e, hs, p->wq, p->wk, p->wv, p->wo, p->w_gate, p->w_up, p->w_down,
                       sv->q, sv->k, sv->v, sv->o, sv->lse, sv->y, sv->u, sv->w, sv->m,
                       gr->de, gr->dwq, gr->dwk, gr->dwv, gr->dwo, gr->dw_gate, gr->dw_up, gr->dw_down, workspace};
  for (const void* q : req) if (!q) return BEAGLE_ERR_NULL;
  if (need_dhs && !gr->dhs) return BEAGLE_ERR_NULL;
  if (p->g_q && (!sv->xq_n || !sv->r_q || !gr->dg_q)) return BEAGLE_ERR_NULL;
  if (p->g_kv && (!sv->xkv_n || !sv->r_kv || !gr->dg_kv)) return BEAGLE_ERR_NULL;
  if (p->g_mlp && (!sv->z || !sv->r_mlp || !gr->dg_mlp)) return BEAGLE_ERR_NULL;
  const void* all[] = {dh, e, hs, p->wq, p->wk, p->wv, p->wo, p->w_gate, p->w_up, p->w_down, p->g_q, p->g_kv, p->g_mlp,
                       sv->xq_n, sv->r_q, sv->xkv_n, sv->r_kv, sv->q, sv->k, sv->v, sv->o, sv->lse, sv->y, sv->z,
                       sv->r_mlp, sv->u, sv->w, sv->m, gr->de, gr->dhs, gr->dwq, gr->dwk, gr->dwv, gr->dwo,
                       gr->dw_gate, gr->dw_up, gr->dw_down, gr->dg_q, gr->dg_kv, gr->dg_mlp};
  for (const void* q : all) if (q && !aligned16(q)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  if (workspace_bytes < beagle_xattn_block_workspace_bytes(desc, p->ffn, ws_kind)) return BEAGLE_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const int64_t Mq = d.Tq, Mk = d.Tk, F = p->ffn;
  const int D = (int)d.D;
  const BlockWs w = block_bwd_layout(d, F);
  char* base = (char*)workspace;
  hs = states_in(d, hs, workspace, beagle_xattn_block_workspace_bytes(desc, p->ffn, ws_kind), s);
  void* dm = base + w.dm; void* dwp = base + w.dw; void* dz = base + w.dz; void* dy = base + w.dy;
  void* dxq_n = base + w.dxq; void* dxkv_n = base + w.dxkv; float* part = (float*)(base + w.part);

  // ---- h = m W_down + y
  run_gemm(d, group1(gemm_nt(dh, p->w_down, dm, Mq, F, d.D)), s, "bwd_mlp_dm");
  run_gemm(d, group1(gemm_tn(sv->m, dh, gr->dw_down, F, d.D, Mq, false)), s, "bwd_mlp_dwdown");
  launch_silu_mul_bwd(d.bf16, dm, sv->u, sv->w, /*du, in place*/ dm, dwp, Mq * F, s);
  const void* du = dm;
  const void* z = p->g_mlp ? sv->z : sv->y;
  {
    GemmGroup g; memset(&g, 0, sizeof(g));
    g.count = 2;
    g.p[0] = gemm_tn(z, du, gr->dw_gate, d.D, F, Mq, false);
    g.p[1] = gemm_tn(z, dwp, gr->dw_up, d.D, F, Mq, false);
    run_gemm(d, g, s, "bwd_mlp_dwgu");
  }
  {
    // dz = du W_gate^T + dw W_up^T; without the MLP's normalisation this is already dy - dh: add dh here
    GemmArgs g = gemm_nt(du, p->w_gate, p->g_mlp ? dz : dy, Mq, d.D, F);
    g.A2 = dwp; g.B2 = p->w_up; g.K2 = (int32_t)F; g.lda2 = F; g.ldb2 = F;
    if (!p->g_mlp) { g.R = dh; g.ldr = d.D; }
    run_gemm(d, group1(g), s, "bwd_mlp_dz");
  }
  if (p->g_mlp)   // dy = dh + dRMSNorm(dz)
    launch_rmsnorm_bwd(d.bf16, dz, sv->y, p->g_mlp, sv->r_mlp, dh, dy, gr->dg_mlp, part, Mq, D, s, "bwd_norm_mlp");

  // ---- y = CrossAttn(xkv, xq) + e
  const bool need_dxkv = need_dhs || p->g_kv;      // the gain's gradient needs dxkv even if dhs is not wanted
  const void* xq = p->g_q ? sv->xq_n : e;
  const void* xkv = p->g_kv ? sv->xkv_n : hs;
  void* dxq_out = p->g_q ? dxq_n : gr->de;
  void* dxkv_out = p->g_kv ? dxkv_n : gr->dhs;
  void* dxp_n = base + w.attn;                      // simulation only: gradient of the normalised predicted states
  if (sim) {
    char* attn_ws = base + w.attn + align_up((size_t)(Mk * d.D) * d.esz);
    xattn_bwd_sim_run(d, need_dxkv, false, dy, xq, xkv, p->g_kv ? sv->xp_n : xpred, p->wq, p->wk, p->wv, p->wo, sv->q, sv->k,
                      sv->v, sv->kp, sv->vp, sv->o, sv->lse, sim_step, dxq_out, dxkv_out, p->g_kv ? dxp_n : gr->dxpred,
                      gr->dwq, gr->dwk, gr->dwv, gr->dwo, attn_ws, p->g_q ? nullptr : dy, s);
  } else {
    xattn_bwd_run(d, need_dxkv, false, dy, xq, xkv, p->wq, p->wk, p->wv, p->wo, sv->q, sv->k, sv->v, sv->o, sv->lse,
                  dxq_out, dxkv_out, gr->dwq, gr->dwk, gr->dwv, gr->dwo, base + w.attn, p->g_q ? nullptr : dy, s);
  }
  if (p->g_q)     // de = dy + dRMSNorm(dxq)
    launch_rmsnorm_bwd(d.bf16, dxq_n, e, p->g_q, sv->r_q, dy, gr->de, gr->dg_q, part, Mq, D, s, "bwd_norm_q");
  if (p->g_kv)
    launch_rmsnorm_bwd(d.bf16, dxkv_n, hs, p->g_kv, sv->r_kv, nullptr, need_dhs ? gr->dhs : dxkv_n, gr->dg_kv, part, Mk, D,
                       s, "bwd_norm_kv");
  if (sim && p->g_kv)   // the same gain normalised the predicted states: its gradient collects both
    launch_rmsnorm_bwd(d.bf16, dxp_n, xpred, p->g_kv, sv->r_p, nullptr, gr->dxpred, gr->dg_kv, part, Mk, D, s,
                       "bwd_norm_pred", true);
  return hip_status();
}
}  // namespace

beagle_status beagle_xattn_block_fwd(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* e, const void* hs, void* h, const beagle_block_saved* sv,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  return block_fwd_impl(desc, p, e, hs, false, nullptr, 0, h, sv, workspace, workspace_bytes, hip_stream);
}
beagle_status beagle_xattn_block_fwd_sim(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* e, const void* hs, const void* xpred, int32_t sim_step, void* h, const beagle_block_saved* sv,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  return block_fwd_impl(desc, p, e, hs, true, xpred, sim_step, h, sv, workspace, workspace_bytes, hip_stream);
}
beagle_status beagle_xattn_block_bwd(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* dh, const void* e, const void* hs, const beagle_block_saved* sv,
    const beagle_block_grads* gr, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return block_bwd_impl(desc, p, dh, e, hs, false, nullptr, 0, sv, gr, workspace, workspace_bytes, hip_stream);
}
beagle_status beagle_xattn_block_bwd_sim(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* dh, const void* e, const void* hs, const void* xpred, int32_t sim_step,
    const beagle_block_saved* sv, const beagle_block_grads* gr, void* workspace, size_t workspace_bytes,
    void* hip_stream) {
  return block_bwd_impl(desc, p, dh, e, hs, true, xpred, sim_step, sv, gr, workspace, workspace_bytes, hip_stream);
}

namespace {
bool decode_weights_ok(const beagle_block_decode_weights* dw) {
  return dw && dw->struct_size == (int32_t)sizeof(beagle_block_decode_weights) && dw->reserved == 0;
}
// shared by the plain entry point (dw == nullptr) and the one on prepared weights
beagle_status block_draft_step_impl(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const beagle_block_decode_weights* dw,
    const void* x_draft, const void* k_cache, const void* v_cache, int32_t n_true, const uint32_t* tree_mask,
    int32_t mask_words, void* h, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_block(desc, p, &d, true);
  if (st != BEAGLE_OK) return st;
  const void* wq = dw ? dw->wq_pk : p->wq;
  const void* wo = dw ? dw->wo_pk : p->wo;
  const void* w_gate = dw ? dw->w_gate_pk : p->w_gate;
  const void* w_up = dw ? dw->w_up_pk : p->w_up;
  const void* w_down = dw ? dw->w_down_pk : p->w_down;
  const void* req[] = {x_draft, k_cache, v_cache, wq, wo, w_gate, w_up, w_down, h, lse, workspace};
  for (const void* q : req) if (!q) return BEAGLE_ERR_NULL;
  const void* all[] = {x_draft, k_cache, v_cache, wq, wo, w_gate, w_up, w_down, p->g_q, p->g_mlp, h, lse};
  for (const void* q : all) if (q && !aligned16(q)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  const int64_t F = p->ffn;
  if (workspace_bytes < beagle_xattn_block_workspace_bytes(desc, p->ffn, BEAGLE_WS_BLOCK_DRAFT)) return BEAGLE_ERR_WORKSPACE;
  if (d.bf16 && !block_mlp_bf16_fits((int32_t)d.D, (int32_t)F)) return BEAGLE_ERR_UNSUPPORTED;
  if (dw && !(d.bf16 && strip_gemm_fits((int32_t)d.S, (int32_t)d.D, (int32_t)d.HD) && strip_gemm_fits((int32_t)d.S, (int32_t)d.HD, (int32_t)d.D) &&
              strip_gemm_fits((int32_t)d.S, (int32_t)F, (int32_t)d.D) && strip_gemm_fits((int32_t)d.S, (int32_t)d.D, (int32_t)F)))
    return BEAGLE_ERR_UNSUPPORTED;
  if (n_true < 0 || n_true > d.L) return BEAGLE_ERR_SHAPE;
  const int64_t T = d.L - n_true;
  if (T > 0) {
    if (!tree_mask) return BEAGLE_ERR_NULL;
    if (((uintptr_t)tree_mask) % 4) return BEAGLE_ERR_ALIGN;
    if (mask_words < (T + 31) / 32) return BEAGLE_ERR_SHAPE;
  } else {
    tree_mask = nullptr; mask_words = 0;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const BlockDraftWs w = block_draft_layout(desc, d, F);
  char* base = (char*)workspace;
  void* y = base + w.y;
  const int D = (int)d.D;

  // y = Attn(RMSNorm(x)) + x
  const void* xn = x_draft;
  // (on packed weights the normalisations ride in the projections: gains in the matrices, row factors in the epilogues)
  if (p->g_q && !dw) { launch_rmsnorm_fwd(d.bf16, x_draft, p->g_q, base + w.xn, (float*)(base + w.rinv), d.S, D, p->rms_eps, s, "draft_norm_q"); xn = base + w.xn; }
  if (d.bf16) {
    DecodeArgs a; memset(&a, 0, sizeof(a));
    a.M = (int32_t)d.S; a.L = (int32_t)d.L; a.H = (int32_t)d.H; a.G = (int32_t)d.G; a.d = (int32_t)d.d;
    a.D = (int32_t)d.D; a.scale = d.scale;
    a.x = xn; a.kc = k_cache; a.vc = v_cache; a.y = y; a.lse = lse; a.ws = base + w.step;
    if (dw) { a.wq_pk = wq; a.wo_pk = wo; a.x_norm_eps = p->g_q ? p->rms_eps : -1.f; } else { a.wq = wq; a.wo = wo; }
    a.tree = tree_mask; a.n_true = n_true; a.tree_words = mask_words;
    a.rope = d.rope ? 1 : 0; a.rope_base = d.rope_base; a.rope_pos = d.rope_pos;
    a.y_res = x_draft;
    launch_decode_bf16(a, s);
  } else {
    char* sb = base + w.step;
    void* q = sb;
    void* o = sb + (size_t)(d.S * d.HD) * d.esz;
    launch_gemm_f32(group1(gemm_nn(xn, p->wq, q, d.S, d.HD, d.D)), s, "draft_proj_q");
    if (d.rope) {
      RopeArgs r = rope_args(d, false);
      rope_add(r, q, d.S, d.rope_pos ? d.S : 1, d.H, (int32_t)d.L, d.rope_pos);
      launch_rope(false, r, s, "draft_rope_q");
    }
    AttnArgs a = attn_args(d);
    a.q = q; a.k = k_cache; a.v = v_cache; a.o = o; a.lse = lse;
    a.tree = tree_mask; a.n_true = n_true; a.tree_words = mask_words;
    launch_attn_fwd_f32(a, s);
    GemmArgs out = gemm_nn(o, p->wo, y, d.S, d.D, d.HD);
    out.R = x_draft; out.ldr = d.D;
    launch_gemm_f32(group1(out), s, "draft_proj_out");
  }
  // h = MLP(RMSNorm(y)) + y
  const void* z = y;
  if (p->g_mlp && !dw) { launch_rmsnorm_fwd(d.bf16, y, p->g_mlp, base + w.z, (float*)(base + w.rinv), d.S, D, p->rms_eps, s, "draft_norm_mlp"); z = base + w.z; }
  if (d.bf16 && dw) {
    launch_block_mlp_strip_bf16(z, w_gate, w_up, w_down, y, h, (int32_t)d.S, (int32_t)d.D, (int32_t)F,
                                p->g_mlp ? p->rms_eps : -1.f, base + w.mlp, s);
  } else if (d.bf16) {
    launch_block_mlp_bf16(z, p->w_gate, p->w_up, p->w_down, y, h, (int32_t)d.S, (int32_t)d.D, (int32_t)F, base + w.mlp, s);
  } else {
    GemmGroup gu; memset(&gu, 0, sizeof(gu));
    gu.count = 2;
    gu.p[0] = gemm_nn(z, p->w_gate, base + w.u, d.S, F, d.D);
    gu.p[1] = gemm_nn(z, p->w_up, base + w.w, d.S, F, d.D);
    launch_gemm_f32(gu, s, "draft_mlp_gate_up");
    launch_silu_mul_fwd(false, base + w.u, base + w.w, base + w.m, d.S * F, s);
    GemmArgs dn = gemm_nn(base + w.m, p->w_down, h, d.S, d.D, F);
    dn.R = y; dn.ldr = d.D;
    launch_gemm_f32(group1(dn), s, "draft_mlp_down");
  }
  return hip_status();
}
}  // namespace

beagle_status beagle_xattn_block_draft_step(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* x_draft, const void* k_cache, const void* v_cache, int32_t n_true, const uint32_t* tree_mask,
    int32_t mask_words, void* h, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return block_draft_step_impl(desc, p, nullptr, x_draft, k_cache, v_cache, n_true, tree_mask, mask_words, h, lse,
                               workspace, workspace_bytes, hip_stream);
}

beagle_status beagle_xattn_block_draft_step_prepared(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const beagle_block_decode_weights* dw, const void* x_draft, const void* k_cache, const void* v_cache,
    int32_t n_true, const uint32_t* tree_mask, int32_t mask_words, void* h, float* lse,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!dw) return BEAGLE_ERR_NULL;
  if (!decode_weights_ok(dw)) return BEAGLE_ERR_SHAPE;
  // the five matrices that dw replaces are not read: the shared checks see dw's in their place
  beagle_block_params q;
  if (!p || p->struct_size != (int32_t)sizeof(q)) return p ? BEAGLE_ERR_SHAPE : BEAGLE_ERR_NULL;
  q = *p;
  q.wq = dw->wq_pk; q.wo = dw->wo_pk; q.w_gate = dw->w_gate_pk; q.w_up = dw->w_up_pk; q.w_down = dw->w_down_pk;
  return block_draft_step_impl(desc, &q, dw, x_draft, k_cache, v_cache, n_true, tree_mask, mask_words, h, lse,
                               workspace, workspace_bytes, hip_stream);
}

beagle_status beagle_xattn_block_prepare_weights(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const beagle_block_decode_weights* dw, void* hip_stream) {
  Dims d; beagle_status st = check_block(desc, p, &d, true);
  if (st != BEAGLE_OK) return st;
  if (!dw) return BEAGLE_ERR_NULL;
  if (!decode_weights_ok(dw)) return BEAGLE_ERR_SHAPE;
  const void* ptrs[] = {p->wq, p->wo, p->w_gate, p->w_up, p->w_down, dw->wq_pk, dw->wo_pk, dw->w_gate_pk, dw->w_up_pk, dw->w_down_pk};
  for (const void* q : ptrs) if (!q) return BEAGLE_ERR_NULL;
  for (const void* q : ptrs) if (!aligned16(q)) return BEAGLE_ERR_ALIGN;
  // the key/value side is optional: both sources and both destinations, or none
  const bool kv = p->wk || p->wv || dw->wk_pk || dw->wv_pk;
  if (kv) {
    const void* kvp[] = {p->wk, p->wv, dw->wk_pk, dw->wv_pk};
    for (const void* q : kvp) if (!q) return BEAGLE_ERR_NULL;
    for (const void* q : kvp) if (!aligned16(q)) return BEAGLE_ERR_ALIGN;
  }
  const int32_t F = p->ffn;
  if (!d.bf16 || F % 128 || d.D % 128 || d.HD % 128 || d.GD % 16) return BEAGLE_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  // the gains of the two normalisations go into the matrices that read the normalised rows
  launch_pack_strips_bf16(p->wq, dw->wq_pk, (int32_t)d.D, (int32_t)d.HD, p->g_q, s);
  launch_pack_strips_bf16(p->wo, dw->wo_pk, (int32_t)d.HD, (int32_t)d.D, nullptr, s);
  launch_pack_strips_bf16(p->w_gate, dw->w_gate_pk, (int32_t)d.D, F, p->g_mlp, s);
  launch_pack_strips_bf16(p->w_up, dw->w_up_pk, (int32_t)d.D, F, p->g_mlp, s);
  launch_pack_strips_bf16(p->w_down, dw->w_down_pk, F, (int32_t)d.D, nullptr, s);
  if (kv) {
    launch_pack_strips_bf16(p->wk, dw->wk_pk, (int32_t)d.D, (int32_t)d.GD, p->g_kv, s);
    launch_pack_strips_bf16(p->wv, dw->wv_pk, (int32_t)d.D, (int32_t)d.GD, p->g_kv, s);
  }
  return hip_status();
}

beagle_status beagle_xattn_block_kv_append_prepared(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const beagle_block_decode_weights* dw, const void* x_new, void* k_cache, void* v_cache, int32_t pos, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  if (!p || !dw) return BEAGLE_ERR_NULL;
  if (p->struct_size != (int32_t)sizeof(beagle_block_params) || p->reserved != 0 || !decode_weights_ok(dw)) return BEAGLE_ERR_SHAPE;
  if (!(p->rms_eps >= 0.f) || isinf(p->rms_eps)) return BEAGLE_ERR_SHAPE;
  const void* ptrs[] = {x_new, dw->wk_pk, dw->wv_pk, k_cache, v_cache};
  for (const void* q : ptrs) if (!q) return BEAGLE_ERR_NULL;
  for (const void* q : ptrs) if (!aligned16(q)) return BEAGLE_ERR_ALIGN;
  if (!(d.bf16 && strip_gemm_fits((int32_t)d.S, (int32_t)d.GD, (int32_t)d.D))) return BEAGLE_ERR_UNSUPPORTED;
  if (pos < 0 || (int64_t)pos + d.S > d.L) return BEAGLE_ERR_SHAPE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  // the key/value normalisation rides in the projection: gain in the packed matrices, row factor in the epilogue
  kv_append_run(d, x_new, dw->wk_pk, dw->wv_pk, k_cache, v_cache, pos, nullptr, s, p->g_kv ? p->rms_eps : -1.f);
  return hip_status();
}

beagle_status beagle_xattn_block_kv_append(const beagle_xattn_desc* desc, const beagle_block_params* p,
    const void* x_new, void* k_cache, void* v_cache, int32_t pos,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims d; beagle_status st = check_desc(desc, true, &d);
  if (st != BEAGLE_OK) return st;
  if (!p) return BEAGLE_ERR_NULL;
  if (p->struct_size != (int32_t)sizeof(beagle_block_params) || p->reserved != 0) return BEAGLE_ERR_SHAPE;
  if (!(p->rms_eps >= 0.f) || isinf(p->rms_eps)) return BEAGLE_ERR_SHAPE;
  const void* ptrs[] = {x_new, p->wk, p->wv, k_cache, v_cache, workspace};
  for (const void* q : ptrs) if (!q) return BEAGLE_ERR_NULL;
  for (const void* q : ptrs) if (!aligned16(q)) return BEAGLE_ERR_ALIGN;
  if (p->g_kv && !aligned16(p->g_kv)) return BEAGLE_ERR_ALIGN;
  if (((uintptr_t)workspace) % WS_ALIGN) return BEAGLE_ERR_ALIGN;
  const size_t need = beagle_xattn_workspace_bytes(desc, BEAGLE_WS_BLOCK_APPEND);
  if (workspace_bytes < need) return BEAGLE_ERR_WORKSPACE;
  if (pos < 0 || (int64_t)pos + d.S > d.L) return BEAGLE_ERR_SHAPE;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  // the normalised copy of the new states and their 1/rms live behind the plain append's own workspace
  char* tail = (char*)workspace + beagle_xattn_workspace_bytes(desc, BEAGLE_WS_APPEND);
  const void* xn = x_new;
  if (p->g_kv) {
    launch_rmsnorm_fwd(d.bf16, x_new, p->g_kv, tail, (float*)(tail + align_up((size_t)(d.S * d.D) * d.esz)), d.S, (int)d.D,
                       p->rms_eps, s, "append_norm_kv");
    xn = tail;
  }
  kv_append_run(d, xn, p->wk, p->wv, k_cache, v_cache, pos, workspace, s);
  return hip_status();
}
