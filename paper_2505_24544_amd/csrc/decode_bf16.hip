// Decode-time draft step (section 4.1, KV-cache paragraph) for bf16, head
// width 128: M <= 64 draft queries per pass against L cached K/V rows, all
// visible.  The step is bound by HBM bandwidth (K/V cache + Wq + Wo are each
// read once), so the kernels are shaped to keep many 16-byte loads in flight
// on every CU; the matrix cores only keep the arithmetic off the critical path.
//
//   (A) skinny_gemm   q_part[ks] = x * Wq[k-slice ks]       grid (N/64, K/512)
//   (B) decode_attn   per (head, key split, 32-query block): each of the 4
//                     waves takes its own run of keys, online softmax per lane
//                     (a lane owns one query, as in the training forward); the
//                     waves' partial (m, l, O) are merged in LDS and written
//                     out unnormalised.  The prologue sums the k-slices of q
//                     and splits q into a bf16 hi + lo pair, so that the scores
//                     (and the LSE) see q at ~16 bits instead of 8.
//   (C) combine       merges the key splits, writes o (bf16) and the LSE
//   (A) skinny_gemm   y_part[ks] = o * Wo[k-slice ks]
//   (E) sum_slices    y = sum_ks y_part[ks]  (bf16)
//
// Everything is deterministic: partial results are summed in a fixed order.
#include "common.h"

namespace beagle {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4_t;
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;

namespace dec {
constexpr int HD = 128;
constexpr float LOG2E = 1.44269504088896340736f;
constexpr int MAXM = 64;               // queries per pass

// ---- (A) skinny GEMM -------------------------------------------------------
constexpr int SG_N = 64;               // output columns per workgroup
constexpr int SG_K = 512;              // k rows per workgroup (128 per wave)
constexpr int SG_LD = SG_N + 32;       // LDS row stride (elements): conflict-free transpose reads

__device__ __forceinline__ uint32_t cvt_pk(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return *(uint32_t*)&b;
}
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
}  // namespace dec

// part[ks][m][n] = sum_{k in slice ks} x[m][k] * W[k][n]     (float)
__global__ __launch_bounds__(256, 1) void skinny_gemm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ W,
                                                             float* __restrict__ part, int M, int N, int K) {
  using namespace dec;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  const int n0 = blockIdx.x * SG_N, ks = blockIdx.y, k0 = ks * SG_K;
  const int mblocks = (M + 31) / 32;

  // all 16 loads of this thread are issued before the first use
  i32x4_t w[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = tid + 256 * i, r = c >> 3, ch = c & 7;
    i32x4_t z = {0, 0, 0, 0};
    w[i] = z;
    if (k0 + r < K) w[i] = *(const i32x4_t*)(W + (int64_t)(k0 + r) * N + n0 + ch * 8);
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = tid + 256 * i, r = c >> 3, ch = c & 7;
    *(i32x4_t*)(smem + r * SG_LD + ch * 8) = w[i];
  }
  __syncthreads();

  f32x16_t acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  const int gi = lane >> 4, r16 = lane & 15;
#pragma unroll
  for (int st = 0; st < 8; ++st) {
    const int kk = wave * 128 + st * 16;
    bf16x8_t xf[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const int m = 32 * mb + (lane & 31);
      bf16x8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
      xf[mb] = z;
      if (mb < mblocks && m < M && k0 + kk + 8 * hf < K) xf[mb] = *(const bf16x8_t*)(x + (int64_t)m * K + k0 + kk + 8 * hf);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const bf16_t* p = smem + (kk + 8 * (gi >> 1) + (r16 >> 2)) * SG_LD + 32 * nb + 16 * (gi & 1) + 4 * (r16 & 3);
      union { struct { s16x4_t a, b; } s; bf16x8_t v; } wf;
      wf.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
      wf.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * SG_LD));
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        if (mb < mblocks) acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xf[mb], acc[nb][mb], 0, 0, 0);
    }
  }
  __syncthreads();                          // every wave is done with the W tile
  // merge the four waves' k-quarters through LDS: red[wave][m][n], n fastest, m rows padded to 68
  float* red = (float*)smem;
  constexpr int RLD = SG_N + 4;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
      if (mb < mblocks) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int m = 32 * mb + (lane & 31), n = 32 * nb + 8 * q + 4 * hf;
          float4 v = {acc[nb][mb][4 * q], acc[nb][mb][4 * q + 1], acc[nb][mb][4 * q + 2], acc[nb][mb][4 * q + 3]};
          *(float4*)(red + (wave * MAXM + m) * RLD + n) = v;
        }
      }
  __syncthreads();
  for (int i = tid; i < M * (SG_N / 4); i += 256) {
    const int m = i / (SG_N / 4), n = (i % (SG_N / 4)) * 4;
    float4 s = *(const float4*)(red + m * RLD + n);
#pragma unroll
    for (int wv = 1; wv < 4; ++wv) {
      const float4 t = *(const float4*)(red + (wv * MAXM + m) * RLD + n);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    *(float4*)(part + ((int64_t)ks * M + m) * N + n0 + n) = s;
  }
}

// y[m][n] = sum_ks part[ks][m][n]  -> bf16
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ part, bf16_t* __restrict__ y,
                                                         int64_t MN, int KS) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= MN) return;
  float4 s = *(const float4*)(part + i);
  for (int k = 1; k < KS; ++k) {
    const float4 t = *(const float4*)(part + (int64_t)k * MN + i);
    s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
  }
  uint2 v = {dec::cvt_pk(s.x, s.y), dec::cvt_pk(s.z, s.w)};
  *(uint2*)(y + i) = v;
}

// ---- (B) split-KV attention -------------------------------------------------
struct DecAttnArgs {
  const float* qpart; int KSq;            // [KSq][M][H*128]
  const bf16_t* kc; const bf16_t* vc;     // [L][G][128]
  float* opart; float* mlpart;            // [H][splits][Mpad][128], [H][splits][Mpad][2]
  int M, Mpad, L, H, G, splits, keys_per_wave;
  float scale;
};

namespace dec {
constexpr int TILE = 64 * HD;                     // one 64-key K or V tile (swizzled rows of 256 B)
constexpr int WAVE_LDS = 2 * TILE;                // K + V, per wave
constexpr int OLD = 33;                           // merge buffer: [wave][c][q], q padded to 33
}  // namespace dec

__global__ __launch_bounds__(256, 1) void decode_attn_kernel(DecAttnArgs a) {
  using namespace dec;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, ql = lane & 31;
  const int h = blockIdx.x, sp = blockIdx.y, mb = blockIdx.z;
  const int g = h / (a.H / a.G);
  const int m = 32 * mb + ql;
  const bool m_ok = m < a.M;
  const int HDt = a.H * HD;

  // ---- q = sum of the projection's k-slices, split into bf16 hi + lo
  bf16x8_t qh[8], qlo[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (m_ok) {
      const float* p = a.qpart + (int64_t)m * HDt + h * HD + 16 * s + 8 * hf;
      for (int k = 0; k < a.KSq; ++k) {
        const float4 t0 = *(const float4*)(p + (int64_t)k * a.M * HDt);
        const float4 t1 = *(const float4*)(p + (int64_t)k * a.M * HDt + 4);
        v[0] += t0.x; v[1] += t0.y; v[2] += t0.z; v[3] += t0.w;
        v[4] += t1.x; v[5] += t1.y; v[6] += t1.z; v[7] += t1.w;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const __bf16 hi = (__bf16)v[i];
      qh[s][i] = hi;
      qlo[s][i] = (__bf16)(v[i] - (float)hi);
    }
  }

  const int jw0 = (sp * 4 + wave) * a.keys_per_wave;
  const int jw1 = min(jw0 + a.keys_per_wave, a.L);
  const bf16_t* Kg = a.kc + (int64_t)g * HD;
  const bf16_t* Vg = a.vc + (int64_t)g * HD;
  const int64_t kvs = (int64_t)a.G * HD;
  bf16_t* ks = smem + wave * WAVE_LDS;
  bf16_t* vs = ks + TILE;
  const float c2 = a.scale * LOG2E;

  f32x16_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
  float mrun = -INFINITY, lrun = 0.f;

  // every wave runs the same number of tiles (tiles past the end of the cache
  // are fully masked), so the barriers below are reached by all waves
#pragma unroll 1
  for (int j0 = jw0; j0 < jw0 + a.keys_per_wave; j0 += 64) {
    // wave-private staging: 32 loads of 16 bytes per lane in flight
    i32x4_t kr[16], vr[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int c = lane + 64 * i, r = c >> 4, ch = c & 15;
      const int j = j0 + r;
      i32x4_t z = {0, 0, 0, 0};
      kr[i] = z; vr[i] = z;
      if (j < jw1) {
        kr[i] = *(const i32x4_t*)(Kg + j * kvs + ch * 8);
        vr[i] = *(const i32x4_t*)(Vg + j * kvs + ch * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int c = lane + 64 * i, r = c >> 4, ch = c & 15;
      *(i32x4_t*)(ks + r * HD + ((ch ^ swz(r)) << 3)) = kr[i];
      *(i32x4_t*)(vs + r * HD + ((ch ^ swz(r)) << 3)) = vr[i];
    }
    __syncthreads();
    f32x16_t st[2];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) st[jb][e] = 0.f;
      const int r = jb * 32 + ql;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const bf16x8_t kf = *(const bf16x8_t*)(ks + r * HD + (((2 * s + hf) ^ swz(r)) << 3));
        st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qh[s], st[jb], 0, 0, 0);
        st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qlo[s], st[jb], 0, 0, 0);
      }
    }
    if (j0 + 64 > jw1) {
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (j0 + 32 * jb + 8 * (e >> 2) + 4 * hf + (e & 3) >= jw1) st[jb][e] = -INFINITY;
    }
    float mx = st[0][0];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[jb][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(mrun, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((mrun - m_safe) * c2);
    const float mc = m_safe * c2;
    float rs = 0.f;
    uint32_t pk[2][8];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(st[jb][e] * c2 - mc);
        const float p1 = __builtin_amdgcn_exp2f(st[jb][e + 1] * c2 - mc);
        rs += p0 + p1;
        pk[jb][e >> 1] = cvt_pk(p0, p1);
      }
    rs += __shfl_xor(rs, 32, 64);
    lrun = lrun * alpha + rs;
    mrun = m_new;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[i][e] *= alpha;
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        union { uint32_t u[4]; bf16x8_t v; } pf;
#pragma unroll
        for (int i = 0; i < 4; ++i) pf.u[i] = pk[jb][4 * t + i];
        const int gi = lane >> 4, r16 = lane & 15;
        const int row = 32 * jb + 16 * t + 4 * (gi >> 1) + (r16 >> 2);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
          const int chunk = 4 * cb + 2 * (gi & 1) + ((r16 & 3) >> 1), sub = 4 * (r16 & 1);
          union { struct { s16x4_t x, y; } s; bf16x8_t v; } vf;
          vf.s.x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vs + row * HD + ((chunk ^ swz(row)) << 3) + sub));
          vf.s.y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vs + (row + 8) * HD + ((chunk ^ swz(row + 8)) << 3) + sub));
          o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[cb], 0, 0, 0);
        }
      }
    __syncthreads();                       // tile fully consumed before it is overwritten
  }

  // ---- merge the four waves (fixed order) and write the split's partial
  float* ob = (float*)smem;                                  // [4][128][OLD]
  float* mlb = ob + 4 * HD * OLD;                            // [4][2][32]
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int c = 32 * cb + 8 * (e >> 2) + 4 * hf + (e & 3);
      ob[(wave * HD + c) * OLD + ql] = o[cb][e];
    }
  if (hf == 0) { mlb[(wave * 2) * 32 + ql] = mrun; mlb[(wave * 2 + 1) * 32 + ql] = lrun; }
  __syncthreads();
  const int64_t pbase = ((int64_t)h * a.splits + sp) * a.Mpad + 32 * mb;
  for (int i = tid; i < 32 * HD; i += 256) {
    const int c = i & (HD - 1), q = i >> 7;
    float mm = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) mm = fmaxf(mm, mlb[(wv * 2) * 32 + q]);
    float acc = 0.f, lt = 0.f;
    if (mm > -INFINITY) {
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) {
        const float sc = __builtin_amdgcn_exp2f((mlb[(wv * 2) * 32 + q] - mm) * c2);
        acc += ob[(wv * HD + c) * OLD + q] * sc;
        lt += mlb[(wv * 2 + 1) * 32 + q] * sc;
      }
    }
    a.opart[(pbase + q) * HD + c] = acc;
    if (c == 0) { a.mlpart[(pbase + q) * 2] = mm; a.mlpart[(pbase + q) * 2 + 1] = lt; }
  }
}

// ---- (C) merge the key splits: o (bf16) and LSE ------------------------------
__global__ __launch_bounds__(128) void decode_combine_kernel(const float* __restrict__ opart, const float* __restrict__ mlpart,
                                                             bf16_t* __restrict__ o, float* __restrict__ lse,
                                                             int lse_stride, int Mpad, int H, int splits, float scale) {
  using namespace dec;
  const int m = blockIdx.x, h = blockIdx.y, c = threadIdx.x;
  const float c2 = scale * LOG2E;
  float mm = -INFINITY;
  for (int s = 0; s < splits; ++s) mm = fmaxf(mm, mlpart[(((int64_t)h * splits + s) * Mpad + m) * 2]);
  float acc = 0.f, lt = 0.f;
  for (int s = 0; s < splits; ++s) {
    const int64_t pb = ((int64_t)h * splits + s) * Mpad + m;
    const float ms = mlpart[pb * 2];
    if (ms == -INFINITY) continue;
    const float sc = __builtin_amdgcn_exp2f((ms - mm) * c2);
    acc += opart[pb * HD + c] * sc;
    lt += mlpart[pb * 2 + 1] * sc;
  }
  const float r = lt > 0.f ? acc / lt : 0.f;
  o[((int64_t)m * H + h) * HD + c] = f32_to_bf16(r);
  if (c == 0) lse[(int64_t)h * lse_stride + m] = lt > 0.f ? mm * scale + logf(lt) : -INFINITY;
}

// ---- host side ----------------------------------------------------------------
namespace {
struct DecLayout {
  int KSq, KSo, splits, keys_per_wave, Mpad;
  size_t qpart, opart, mlpart, o, ypart, total;
};
size_t up256(size_t v) { return (v + 255) / 256 * 256; }
DecLayout dec_layout(int M, int L, int H, int d, int D) {
  DecLayout w;
  const int Mp = M < dec::MAXM ? M : dec::MAXM;             // queries per pass
  const int64_t HDt = (int64_t)H * d;
  w.KSq = (D + dec::SG_K - 1) / dec::SG_K;
  w.KSo = (int)((HDt + dec::SG_K - 1) / dec::SG_K);
  int splits = (L + 255) / 256;
  if (splits > 64) splits = 64;
  if (splits < 1) splits = 1;
  const int per_split = (L + splits - 1) / splits;
  w.keys_per_wave = ((per_split + 3) / 4 + 63) / 64 * 64;
  w.splits = (L + 4 * w.keys_per_wave - 1) / (4 * w.keys_per_wave);
  w.Mpad = (Mp + 31) / 32 * 32;
  size_t o = 0;
  w.qpart = o; o += up256((size_t)w.KSq * Mp * HDt * 4);
  w.opart = o; o += up256((size_t)H * w.splits * w.Mpad * dec::HD * 4);
  w.mlpart = o; o += up256((size_t)H * w.splits * w.Mpad * 2 * 4);
  w.o = o; o += up256((size_t)Mp * HDt * 2);
  w.ypart = o; o += up256((size_t)w.KSo * Mp * D * 4);
  w.total = o;
  return w;
}
}  // namespace

size_t decode_bf16_ws_bytes(int32_t M, int32_t L, int32_t H, int32_t d, int32_t D) {
  return dec_layout(M, L, H, d, D).total;
}

void launch_decode_bf16(const DecodeArgs& a, hipStream_t s) {
  using namespace dec;
  const DecLayout w = dec_layout(a.M, a.L, a.H, a.d, a.D);
  const int HDt = a.H * HD;
  char* base = (char*)a.ws;
  float* qpart = (float*)(base + w.qpart);
  float* opart = (float*)(base + w.opart);
  float* mlpart = (float*)(base + w.mlpart);
  bf16_t* o = (bf16_t*)(base + w.o);
  float* ypart = (float*)(base + w.ypart);
  constexpr size_t sg_smem = (size_t)SG_K * SG_LD * sizeof(bf16_t);
  constexpr size_t at_smem = (size_t)4 * WAVE_LDS * sizeof(bf16_t);
  static_assert(sg_smem >= 4 * MAXM * (SG_N + 4) * sizeof(float), "merge buffer must fit in the W tile");
  static_assert(at_smem >= (4 * HD * OLD + 4 * 2 * 32) * sizeof(float), "merge buffer must fit in the K/V tiles");
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)skinny_gemm_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sg_smem);
    (void)hipFuncSetAttribute((const void*)decode_attn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)at_smem);
    attr_set = true;
  }
  for (int m0 = 0; m0 < a.M; m0 += MAXM) {
    const int Mp = a.M - m0 < MAXM ? a.M - m0 : MAXM;
    const bf16_t* x = (const bf16_t*)a.x + (int64_t)m0 * a.D;
    {
      ProfScope ps("draft_proj_q", s);
      hipLaunchKernelGGL(skinny_gemm_kernel, dim3(HDt / SG_N, w.KSq), dim3(256), sg_smem, s,
                         x, (const bf16_t*)a.wq, qpart, Mp, HDt, a.D);
    }
    {
      DecAttnArgs t;
      t.qpart = qpart; t.KSq = w.KSq; t.kc = (const bf16_t*)a.kc; t.vc = (const bf16_t*)a.vc;
      t.opart = opart; t.mlpart = mlpart; t.M = Mp; t.Mpad = w.Mpad; t.L = a.L; t.H = a.H; t.G = a.G;
      t.splits = w.splits; t.keys_per_wave = w.keys_per_wave; t.scale = a.scale;
      ProfScope ps("draft_attn", s);
      hipLaunchKernelGGL(decode_attn_kernel, dim3(a.H, w.splits, (Mp + 31) / 32), dim3(256), at_smem, s, t);
    }
    {
      ProfScope ps("draft_combine", s);
      hipLaunchKernelGGL(decode_combine_kernel, dim3(Mp, a.H), dim3(128), 0, s, opart, mlpart, o,
                         a.lse + m0, a.M, w.Mpad, a.H, w.splits, a.scale);
    }
    {
      ProfScope ps("draft_proj_out", s);
      hipLaunchKernelGGL(skinny_gemm_kernel, dim3(a.D / SG_N, w.KSo), dim3(256), sg_smem, s,
                         (const bf16_t*)o, (const bf16_t*)a.wo, ypart, Mp, a.D, HDt);
    }
    {
      ProfScope ps("draft_sum_out", s);
      const int64_t MN = (int64_t)Mp * a.D;
      hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((MN / 4 + 255) / 256)), dim3(256), 0, s,
                         ypart, (bf16_t*)a.y + (int64_t)m0 * a.D, MN, w.KSo);
    }
  }
}

}  // namespace beagle
