// Shared between the translation units that hold the C-ABI entry points: the validated view of a descriptor,
// workspace layouts and the host-side sequences of launches that several entry points reuse.  Not part of the
// public interface.
#pragma once
#include "../../include/beagle_xattn.h"
#include "common.h"

namespace beagle {
namespace detail {

constexpr size_t WS_ALIGN = 256;

inline size_t align_up(size_t v) { return (v + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }
inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

struct Dims {
  int64_t B, S, L, D, H, G, d, HD, GD;
  size_t esz;
  bool bf16;
  float scale;
  MaskParams mask;
  const int32_t* eps_b;   // per-entry window offsets (device) or null
  bool rope; float rope_base; const int32_t* rope_pos;
  int64_t Tq, Tk;          // query / key rows in total: B*S, B*L, or the packed row counts
  const int32_t* cu_q; const int32_t* cu_kv;   // packed batches (device, B+1 entries each) or null
  bool kv_f16;             // the key/value source states arrive as IEEE half
};

struct BwdWs { size_t dO, dQ, dK, dV, delta, dwpart, attn, total; };   // dwpart: see split_kv_wgrad

beagle_status check_desc(const beagle_xattn_desc* c, bool draft, Dims* out);
BwdWs bwd_layout(const Dims& d);
bool split_kv_wgrad(const Dims& d);
AttnArgs attn_args(const Dims& d);
// C[M,N] = A[M,K] B with B stored [K,N]; ... = A W^T with W stored [N,K]; ... = X^T Y with X [K,M], Y [K,N]
GemmArgs gemm_nn(const void* A, const void* W, void* C, int64_t M, int64_t N, int64_t K);
GemmArgs gemm_nt(const void* A, const void* W, void* C, int64_t M, int64_t N, int64_t K);
GemmArgs gemm_tn(const void* X, const void* Y, void* C, int64_t M, int64_t N, int64_t K, bool c_f32);
GemmGroup group1(const GemmArgs& a);
void run_gemm(const Dims& d, const GemmGroup& g, hipStream_t s, const char* name);
beagle_status hip_status();
size_t states_ws(const Dims& d);
const void* states_in(const Dims& d, const void* xkv, void* workspace, size_t need, hipStream_t s);
RopeArgs rope_args(const Dims& d, bool inverse);
void rope_add(RopeArgs& r, void* x, int64_t rows, int64_t period, int64_t heads, int32_t pos0, const int32_t* pos,
              const int32_t* cu = nullptr);
void xattn_fwd_run(const Dims& d, const void* xq, const void* xkv, const void* wq, const void* wk, const void* wv,
                   const void* wo, void* y, float* lse, void* q_save, void* k_save, void* v_save, void* o_save,
                   const void* y_res, hipStream_t s);
void xattn_bwd_run(const Dims& d, bool need_dxkv, bool wf32, const void* dy, const void* xq, const void* xkv,
                   const void* wq, const void* wk, const void* wv, const void* wo, const void* q_save,
                   const void* k_save, const void* v_save, const void* o_save, const float* lse, void* dxq,
                   void* dxkv, void* dwq, void* dwk, void* dwv, void* dwo, char* base, const void* dxq_res,
                   hipStream_t s);
void xattn_fwd_sim_run(const Dims& d, const void* xq, const void* xkv, const void* xpred, const void* wq, const void* wk,
                       const void* wv, const void* wo, int32_t sim_step, void* y, float* lse, void* q_save, void* k_save,
                       void* v_save, void* kp_save, void* vp_save, void* o_save, const void* y_res, hipStream_t s);
void xattn_bwd_sim_run(const Dims& d, bool need_dxkv, bool wf32, const void* dy, const void* xq, const void* xkv,
                       const void* xpred, const void* wq, const void* wk, const void* wv, const void* wo,
                       const void* q_save, const void* k_save, const void* v_save, const void* kp_save,
                       const void* vp_save, const void* o_save, const float* lse, int32_t sim_step, void* dxq, void* dxkv,
                       void* dxpred, void* dwq, void* dwk, void* dwv, void* dwo, char* base, const void* dxq_res,
                       hipStream_t s);
// packed_norm_eps: NaN = wk, wv in their stored layout; otherwise they are packed for strip_gemm_kernel, with (>= 0) or
// without (< 0) the row factor of an RMSNorm in front of them (its gain folded into the matrices)
void kv_append_run(const Dims& d, const void* x_new, const void* wk, const void* wv, void* k_cache, void* v_cache,
                   int32_t pos, void* workspace, hipStream_t s, float packed_norm_eps = __builtin_nanf(""));

}  // namespace detail
}  // namespace beagle
