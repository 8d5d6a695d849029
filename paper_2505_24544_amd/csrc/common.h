// Shared declarations of the HIP sources: bf16 storage helpers, the launch
// profiler hooks, and the internal launcher prototypes.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "mask_index.h"

namespace beagle {

typedef uint16_t bf16_t;   // storage type: raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(((uint32_t)v) << 16);
}
// round-to-nearest-even, NaN stays NaN: the hardware conversion (v_cvt_pk_bf16_f32), two values per instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(float)))) float cvt_f32x2_t;
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 cvt_bf16x2_t;
  const cvt_f32x2_t f = {lo, hi};
  const cvt_bf16x2_t b = __builtin_convertvector(f, cvt_bf16x2_t);
  return *(const uint32_t*)&b;
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// ---- launch profiler (see beagle_xattn_profile_* in the public header) ----
void prof_before(const char* name, hipStream_t s);
void prof_after(hipStream_t s);
struct ProfScope {
  hipStream_t s;
  ProfScope(const char* name, hipStream_t st) : s(st) { prof_before(name, st); }
  ~ProfScope() { prof_after(s); }
};

// ---- GEMM:  C[M,N] (+)= op(A) * op(B), float accumulation -----------------
// a_kmajor: A is stored [M,K] (k fastest, leading dim lda) else [K,M].
// b_kmajor: B is stored [N,K] (k fastest, leading dim ldb) else [K,N].
// C is row-major [M,N] with leading dim ldc.  accumulate: C += instead of C =.
// An optional second k-segment (A2, B2, K2; same storage orders and leading
// dims lda2/ldb2) is contracted into the same C:  C = A*B + A2*B2.
struct GemmArgs {
  const void* A; const void* B; void* C;
  int32_t M, N, K;
  int64_t lda, ldb, ldc;
  int32_t a_kmajor, b_kmajor;
  int32_t c_is_f32;      // bf16 inputs only: write float instead of bf16
  const void* A2; const void* B2;
  int32_t K2;
  int64_t lda2, ldb2;
  const void* R;         // optional residual added in the epilogue: C = A B (+ A2 B2) + R; storage type of A,
  int64_t ldr;           // row stride ldr; not with c_is_f32
};
// Up to 4 independent GEMMs in one launch (they share one grid).
struct GemmGroup {
  int32_t count;
  GemmArgs p[4];
};
void launch_gemm_f32(const GemmGroup& g, hipStream_t s, const char* name);
void launch_gemm_bf16(const GemmGroup& g, hipStream_t s, const char* name);
// whether the MFMA kernel covers the group (storage orders, k granularity, 32-bit operand extents)
bool gemm_bf16_supported(const GemmGroup& g);
// out[i] = a[i] + b[i] for up to two (a, b, out) triples of n floats each in one launch (n % 4 == 0); out is bf16 or
// float.  The two halves of a GEMM whose contraction was split over two problems of a group.
struct SumPairArgs { const float* a[2]; const float* b[2]; void* out[2]; int32_t count; };
void launch_sum_pairs(const SumPairArgs& p, int64_t n, bool out_f32, hipStream_t s, const char* name);

// ---- draft block around the attention (section 4.1, Eq. 1): streaming kernels ----
constexpr int RMS_BWD_MAX_PARTS = 1024;      // workgroups (= column-partial rows) of the RMSNorm backward
constexpr int RMS_MAX_D = 12288;             // its column partials live in LDS: 4 * D bytes
int rmsnorm_bwd_parts(int64_t rows);
void launch_rmsnorm_fwd(bool bf16, const void* x, const void* gain, void* out, float* rinv, int64_t rows, int D,
                        float eps, hipStream_t s, const char* name);
// dx = d rmsnorm / dx applied to dout (+ add if given); dgain [D] float; part: rmsnorm_bwd_parts(rows) * D floats
void launch_rmsnorm_bwd(bool bf16, const void* dout, const void* x, const void* gain, const float* rinv,
                        const void* add, void* dx, float* dgain, float* part, int64_t rows, int D, hipStream_t s,
                        const char* name, bool accumulate = false);   // accumulate: dgain += instead of =
// n IEEE half values -> the storage type (n % 8 == 0)
void launch_cvt_f16(bool bf16, const void* in, void* out, int64_t n, hipStream_t s);
void launch_silu_mul_fwd(bool bf16, const void* u, const void* w, void* m, int64_t n, hipStream_t s);
void launch_silu_mul_bwd(bool bf16, const void* dm, const void* u, const void* w, void* du, void* dw, int64_t n,
                         hipStream_t s);

// ---- rotary position embedding, in place, of up to three [rows, heads, d] tensors in one launch ----
// Row r of tensor t stands at position pos[t] ? pos[t][r % period[t]] : pos0[t] + r % period[t].
struct RopeArgs {
  int32_t n;                    // tensors
  void* x[3];
  int64_t rows[3];
  int32_t period[3], heads[3], pos0[3];
  const int32_t* pos[3];        // device, or null
  const int32_t* cu[3];         // packed batch: row r of tensor t is row r - cu[b] of the entry b that holds it
  int32_t nb;                   // entries (cu has nb + 1 values)
  int32_t d;                    // head width, d % 4 == 0, d <= 128
  float base;
  int32_t inverse;              // rotate by -angle (gradients)
};
void launch_rope(bool bf16, const RopeArgs& r, hipStream_t s, const char* name);

// ---- attention -------------------------------------------------------------
struct AttnArgs {
  int32_t B, S, L, H, G, d;
  float scale;
  MaskParams mask;
  const int32_t* eps_b;                           // per batch entry window offsets (device, [B]) or null
  // packed batches (cu_q != null): entry b owns query rows cu_q[b] .. cu_q[b+1]-1 of the Tq packed rows and key
  // rows cu_kv[b] .. cu_kv[b+1]-1 of the Tk; S and L are then the longest lengths (they size the grids)
  const int32_t* cu_q; const int32_t* cu_kv;
  int32_t Tq, Tk;
  const void* q; const void* k; const void* v;   // [B,S,H,d], [B,L,G,d] x2
  void* o; float* lse;                            // [B,S,H,d], [B,H,S]
  // backward only
  const void* dout;                               // dO [B,S,H,d]
  void* dq; void* dk; void* dv;                   // [B,S,H,d], [B,L,G,d] x2
  float* delta;                                   // [B,H,S]
  float* nlse2;                                   // [B,H,S] -log2(e) * LSE, from the dQ kernel to the dK/dV kernel (bf16 path)
  // draft-tree decode only: keys >= n_true are visible to query p iff bit (j - n_true) of row p is set
  const uint32_t* tree; int32_t n_true, tree_words;
};

// Kernel arguments reach the scalar registers through loads that the compiler places where a field is first used: in
// the attention kernels' prologues that made eight trips to the constant cache in a row (some 2 000 cycles per
// workgroup, measured).  Naming every field in one empty statement at the top makes it one trip.
__device__ __forceinline__ void args_at_hand(const AttnArgs& a) {
  asm volatile("" :: "s"(a.B), "s"(a.S), "s"(a.L), "s"(a.H), "s"(a.G), "s"(a.scale), "s"(a.mask.k), "s"(a.mask.eps),
               "s"(a.mask.seq_kv), "s"(a.mask.all_visible), "s"(a.eps_b), "s"(a.cu_q), "s"(a.cu_kv), "s"(a.Tq), "s"(a.Tk),
               "s"(a.q), "s"(a.k), "s"(a.v), "s"(a.o), "s"(a.lse), "s"(a.dout), "s"(a.dq), "s"(a.dk), "s"(a.dv),
               "s"(a.delta), "s"(a.nlse2));
}

// Where batch entry b lives: its lengths, its first query / key row, the offset of its LSE / delta entry (head 0,
// query 0) and the distance between heads there.  Batched layout: rows b*S .., lse [B,H,S].  Packed layout: rows
// from cu_q / cu_kv, lse [H,Tq].  Offsets that do not describe rows inside the packed tensors are clamped, so
// that a wrong cu array gives wrong numbers but never an access outside the buffers.
struct SeqView { int32_t S, L; int64_t q0, kv0, lse0, lse_hs; };
__device__ __forceinline__ SeqView seq_view(const AttnArgs& a, int b) {
  SeqView v;
  if (!a.cu_q) {
    v.S = a.S; v.L = a.L; v.q0 = (int64_t)b * a.S; v.kv0 = (int64_t)b * a.L;
    v.lse0 = (int64_t)b * a.H * a.S; v.lse_hs = a.S;
    return v;
  }
  const int32_t q0 = min(max(a.cu_q[b], 0), a.Tq), k0 = min(max(a.cu_kv[b], 0), a.Tk);
  v.S = min(max(a.cu_q[b + 1] - q0, 0), min(a.S, a.Tq - q0));
  v.L = min(max(a.cu_kv[b + 1] - k0, 0), min(a.L, a.Tk - k0));
  v.q0 = q0; v.kv0 = k0; v.lse0 = q0; v.lse_hs = a.Tq;
  return v;
}

// The mask of batch entry b: the shared parameters, with the entry's own window offset if offsets were given
// and its own key count in a packed batch.
__device__ __forceinline__ MaskParams sample_mask(const AttnArgs& a, int b) {
  MaskParams m = a.mask;
  if (a.cu_q) m.seq_kv = seq_view(a, b).L;
  if (a.eps_b) {
    const int32_t e = a.eps_b[b] % m.k;
    m.eps = e < 0 ? e + m.k : e;
  }
  return m;
}
// Late-stage simulation: the band of predicted keys of every query, merged into / differentiated
// against the result of the masked attention over the true keys.
struct SimArgs {
  AttnArgs a;                       // q, o, lse (in/out), dout, dq (in/out), delta as in the main kernels
  const void* kp; const void* vp;   // [B,L,G,d] predicted-state keys / values
  void* dkp; void* dvp;             // [B,L,G,d]
  int32_t t;                        // simulation step, 0 <= t
  int32_t is_bf16;
};
void launch_sim_band_fwd(const SimArgs& s, hipStream_t st);
void launch_sim_band_bwd(const SimArgs& s, hipStream_t st);
void launch_sim_save(const void* h, void* xpred, int B, int L, int64_t row_bytes, int k, int eps, const int32_t* eps_b,
                     int t, const int32_t* cu, int total, hipStream_t st);
// streaming variants for bf16 storage (head width 128), chosen by the two launchers above
void launch_sim_band_fwd_bf16(const SimArgs& s, hipStream_t st);
void launch_sim_band_bwd_bf16(const SimArgs& s, hipStream_t st);
void launch_attn_fwd_f32(const AttnArgs& a, hipStream_t s);
void launch_attn_bwd_f32(const AttnArgs& a, hipStream_t s);
void launch_attn_fwd_bf16(const AttnArgs& a, hipStream_t s);
void launch_attn_bwd_bf16(const AttnArgs& a, void* ws, hipStream_t s);
size_t attn_bwd_bf16_ws_bytes(const AttnArgs& a);

// ---- decode (bf16): split-KV attention of M queries over L cache rows ------
struct DecodeArgs {
  int32_t M, L, H, G, d, D;
  float scale;
  const void* x; const void* kc; const void* vc; const void* wq; const void* wo;
  void* y; float* lse;
  void* ws;
  // draft tree (tree == nullptr: every cache row is visible to every query)
  const uint32_t* tree; int32_t n_true, tree_words;
  // rotary embedding of the queries (rope != 0): positions rope_pos[m] (device) or all at L
  int32_t rope; float rope_base; const int32_t* rope_pos;
  const void* y_res;   // optional residual added to y (storage type, [M,D])
  // optional: wq / wo packed for strip_gemm_kernel; then wq / wo is not read (needs strip_gemm_fits for M and its shape)
  const void* wq_pk; const void* wo_pk;
  float x_norm_eps;    // with wq_pk: >= 0 applies RMSNorm's row factor to x inside the query projection (gain folded into wq_pk)
};
bool strip_gemm_fits(int32_t M, int32_t N, int32_t K);
// W [K][N] row-major -> the packed layout that strip_gemm_kernel streams (K % 128 == 0, N % 16 == 0)
void launch_pack_strips_bf16(const void* in, void* out, int32_t K, int32_t N, const void* gain, hipStream_t s);
size_t decode_bf16_ws_bytes(int32_t M, int32_t L, int32_t H, int32_t d, int32_t D);
void launch_decode_bf16(const DecodeArgs& a, hipStream_t s);
void launch_read_probe(const void* buf, int64_t bytes, int wgs, uint32_t* sink, hipStream_t s);
void launch_clock_probe(uint64_t* out, hipStream_t s);
size_t kv_append_bf16_ws_bytes(int32_t n, int32_t N, int32_t K);
bool kv_append_bf16_fits(int32_t n, int32_t N, int32_t K);
// feed-forward layer for a handful of rows: h = (silu(z W_gate) * (z W_up)) W_down + y_res
size_t block_mlp_bf16_ws_bytes(int32_t M, int32_t D, int32_t F);
bool block_mlp_bf16_fits(int32_t D, int32_t F);
void launch_block_mlp_bf16(const void* z, const void* w_gate, const void* w_up, const void* w_down, const void* y_res,
                           void* h, int32_t M, int32_t D, int32_t F, void* ws, hipStream_t s);
// the same on packed weights: two strip launches, gate fused;
// needs strip_gemm_fits(M, F, D) and strip_gemm_fits(M, D, F); ws: M * F bf16
void launch_kv_append_strip_bf16(const void* x, const void* wk_pk, const void* wv_pk, void* kdst, void* vdst, int32_t n,
                                 int32_t N, int32_t K, float norm_eps, hipStream_t s);
void launch_block_mlp_strip_bf16(const void* z, const void* w_gate_pk, const void* w_up_pk, const void* w_down_pk,
                                 const void* y_res, void* h, int32_t M, int32_t D, int32_t F, float z_norm_eps, void* ws,
                                 hipStream_t s);
void launch_kv_append_bf16(const void* x, const void* wk, const void* wv, void* kdst, void* vdst, int32_t n, int32_t N,
                           int32_t K, void* ws, hipStream_t s);

}  // namespace beagle
