// Scalar-FMA path: reference-grade kernels, templated on the storage type
// (float, or bfloat16 bits that are widened on load and rounded on store).
// Plain FMA arithmetic, float accumulation, accurate expf/logf.  This is the
// path of io_dtype == BEAGLE_F32 (parity at 1e-5, not speed); bf16 problems run
// on the MFMA kernels only -- what those do not cover is refused by the entry
// points, never routed here.
#include "common.h"

namespace beagle {

template <typename T> struct Io;
template <> struct Io<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Io<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// --------------------------------------------------------------------------
// GEMM: 64x64 output tile, 16-deep k slices through LDS, 4x4 per thread.
// TI: storage type of A and B; TO: storage type of C.
// --------------------------------------------------------------------------
constexpr int FT = 64, FK = 16;

template <typename TI, typename TO>
__global__ __launch_bounds__(256) void gemm_scalar_kernel(GemmGroup grp) {
  __shared__ float As[FK][FT + 4];
  __shared__ float Bs[FK][FT + 4];
  // blockIdx.z selects the problem; blocks outside its tile grid leave
  const GemmArgs& g = grp.p[blockIdx.z];
  const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;
  if (m0 >= g.M || n0 >= g.N) return;
  TO* __restrict__ C = (TO*)g.C;
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int seg = 0; seg < 2; ++seg) {
    const TI* __restrict__ A = (const TI*)(seg ? g.A2 : g.A);
    const TI* __restrict__ B = (const TI*)(seg ? g.B2 : g.B);
    const int K = seg ? g.K2 : g.K;
    const int64_t lda = seg ? g.lda2 : g.lda, ldb = seg ? g.ldb2 : g.ldb;
    if (A == nullptr || K <= 0) continue;
    for (int k0 = 0; k0 < K; k0 += FK) {
      for (int i = tid; i < FT * FK; i += 256) {
        int m, kk;   // element (m, kk) of the A tile; the fastest-varying index
                     // follows the storage order so that loads coalesce
        if (g.a_kmajor) { kk = i % FK; m = i / FK; } else { m = i % FT; kk = i / FT; }
        int gm = m0 + m, gk = k0 + kk;
        float v = 0.f;
        if (gm < g.M && gk < K)
          v = Io<TI>::ld(g.a_kmajor ? A + (int64_t)gm * lda + gk : A + (int64_t)gk * lda + gm);
        As[kk][m] = v;
        int n, kb;
        if (g.b_kmajor) { kb = i % FK; n = i / FK; } else { n = i % FT; kb = i / FT; }
        int gn = n0 + n, gkb = k0 + kb;
        float w = 0.f;
        if (gn < g.N && gkb < K)
          w = Io<TI>::ld(g.b_kmajor ? B + (int64_t)gn * ldb + gkb : B + (int64_t)gkb * ldb + gn);
        Bs[kb][n] = w;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < FK; ++kk) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn >= g.N) continue;
      float r = 0.f;
      if (g.R) r = Io<TI>::ld((const TI*)g.R + (int64_t)gm * g.ldr + gn);
      Io<TO>::st(C + (int64_t)gm * g.ldc + gn, acc[i][j] + r);
    }
  }
}

template <typename TI>
static void gemm_scalar_launch(const GemmGroup& grp, hipStream_t s, const char* name) {
  int mt = 0, nt = 0;
  for (int i = 0; i < grp.count; ++i) {
    mt = max(mt, (grp.p[i].M + FT - 1) / FT);
    nt = max(nt, (grp.p[i].N + FT - 1) / FT);
  }
  if (mt == 0 || nt == 0) return;
  bool f32out = grp.p[0].c_is_f32;
  ProfScope ps(name, s);
  dim3 grid(nt, mt, grp.count);
  if (sizeof(TI) == 4 || f32out) hipLaunchKernelGGL((gemm_scalar_kernel<TI, float>), grid, dim3(256), 0, s, grp);
  else hipLaunchKernelGGL((gemm_scalar_kernel<TI, bf16_t>), grid, dim3(256), 0, s, grp);
}

void launch_gemm_f32(const GemmGroup& g, hipStream_t s, const char* name) { gemm_scalar_launch<float>(g, s, name); }

// --------------------------------------------------------------------------
// Attention, one wavefront per (b, h, p) query row (forward, dQ) or per
// (b, g, j) key row (dK, dV).  Keys/queries are taken 64 at a time: each lane
// owns one of them for the dot products, then the lanes switch to owning head
// channels for the weighted sums.
// --------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const T* __restrict__ row, int d) {
  float s = 0.f;
  for (int c = 0; c < d; c += 4) {
    s = fmaf(a_lds[c], Io<T>::ld(row + c), s);
    s = fmaf(a_lds[c + 1], Io<T>::ld(row + c + 1), s);
    s = fmaf(a_lds[c + 2], Io<T>::ld(row + c + 2), s);
    s = fmaf(a_lds[c + 3], Io<T>::ld(row + c + 3), s);
  }
  return s;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_scalar_kernel(AttnArgs a) {
  __shared__ float qs[128];
  __shared__ float pch[64];
  const int p = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const SeqView sv = seq_view(a, b);
  if (p >= sv.S) return;                               // packed batch: a shorter entry
  const int d = a.d, g = h / (a.H / a.G);
  const T* Q = (const T*)a.q + ((sv.q0 + p) * a.H + h) * d;
  const T* K = (const T*)a.k + (sv.kv0 * a.G + g) * d;
  const T* V = (const T*)a.v + (sv.kv0 * a.G + g) * d;
  const int64_t kvs = (int64_t)a.G * d;
  T* O = (T*)a.o + ((sv.q0 + p) * a.H + h) * d;
  const int64_t li = sv.lse0 + h * sv.lse_hs + p;
  const int n = row_limit(p, sample_mask(a, b));
  for (int c = lane; c < d; c += 64) qs[c] = Io<T>::ld(Q + c);
  __syncthreads();
  if (n == 0) {
    for (int c = lane; c < d; c += 64) Io<T>::st(O + c, 0.f);
    if (lane == 0) a.lse[li] = -INFINITY;
    return;
  }
  // draft-tree decode: keys at or past n_true are visible only where the query's tree row has a bit
  const uint32_t* trow = a.tree ? a.tree + (int64_t)p * a.tree_words : nullptr;
  auto visible = [&](int j) {
    if (trow == nullptr || j < a.n_true) return true;
    const int t = j - a.n_true;
    return ((trow[t >> 5] >> (t & 31)) & 1u) != 0;
  };
  // pass A: row max and sum of exponentials, online per lane, then merged
  float m = -INFINITY, l = 0.f;
  for (int j = lane; j < n; j += 64) {
    if (!visible(j)) continue;
    float s = a.scale * dot_row(qs, K + j * kvs, d);
    float mn = fmaxf(m, s);
    l = l * expf(m - mn) + expf(s - mn);
    m = mn;
  }
  const float mw = wave_max(m);
  if (mw == -INFINITY) {                       // the tree hides every row from this query
    for (int c = lane; c < d; c += 64) Io<T>::st(O + c, 0.f);
    if (lane == 0) a.lse[li] = -INFINITY;
    return;
  }
  l = wave_sum(m == -INFINITY ? 0.f : l * expf(m - mw));
  const float lse = mw + logf(l);
  // pass B: probabilities from the final lse, weighted sum of V
  float acc0 = 0.f, acc1 = 0.f;
  for (int j0 = 0; j0 < n; j0 += 64) {
    int j = j0 + lane;
    pch[lane] = (j < n && visible(j)) ? expf(a.scale * dot_row(qs, K + j * kvs, d) - lse) : 0.f;
    __syncthreads();
    int cnt = min(64, n - j0);
    for (int jj = 0; jj < cnt; ++jj) {
      const T* vr = V + (int64_t)(j0 + jj) * kvs;
      float pj = pch[jj];
      if (lane < d) acc0 = fmaf(pj, Io<T>::ld(vr + lane), acc0);
      if (lane + 64 < d) acc1 = fmaf(pj, Io<T>::ld(vr + lane + 64), acc1);
    }
    __syncthreads();
  }
  if (lane < d) Io<T>::st(O + lane, acc0);
  if (lane + 64 < d) Io<T>::st(O + lane + 64, acc1);
  if (lane == 0) a.lse[li] = lse;
}

// delta[b,h,p] = sum_c dO*O ; dQ_p = scale * sum_j dS_pj K_j
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_scalar_kernel(AttnArgs a) {
  __shared__ float qs[128];
  __shared__ float dos[128];
  __shared__ float dsch[64];
  const int p = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const SeqView sv = seq_view(a, b);
  if (p >= sv.S) return;                               // packed batch: a shorter entry
  const int d = a.d, g = h / (a.H / a.G);
  const int64_t row = ((sv.q0 + p) * a.H + h) * d;
  const T* Q = (const T*)a.q + row;
  const T* O = (const T*)a.o + row;
  const T* dO = (const T*)a.dout + row;
  T* dQ = (T*)a.dq + row;
  const T* K = (const T*)a.k + (sv.kv0 * a.G + g) * d;
  const T* V = (const T*)a.v + (sv.kv0 * a.G + g) * d;
  const int64_t kvs = (int64_t)a.G * d;
  const int64_t li = sv.lse0 + h * sv.lse_hs + p;
  const int n = row_limit(p, sample_mask(a, b));
  float part = 0.f;
  for (int c = lane; c < d; c += 64) {
    qs[c] = Io<T>::ld(Q + c);
    float t = Io<T>::ld(dO + c);
    dos[c] = t;
    part = fmaf(t, Io<T>::ld(O + c), part);
  }
  const float delta = wave_sum(part);
  if (lane == 0) a.delta[li] = delta;
  __syncthreads();
  if (n == 0) { for (int c = lane; c < d; c += 64) Io<T>::st(dQ + c, 0.f); return; }
  const float lse = a.lse[li];
  float acc0 = 0.f, acc1 = 0.f;
  for (int j0 = 0; j0 < n; j0 += 64) {
    int j = j0 + lane;
    float ds = 0.f;
    if (j < n) {
      float pj = expf(a.scale * dot_row(qs, K + j * kvs, d) - lse);
      float dp = dot_row(dos, V + j * kvs, d);
      ds = pj * (dp - delta);
    }
    dsch[lane] = ds;
    __syncthreads();
    int cnt = min(64, n - j0);
    for (int jj = 0; jj < cnt; ++jj) {
      const T* kr = K + (int64_t)(j0 + jj) * kvs;
      float w = dsch[jj];
      if (lane < d) acc0 = fmaf(w, Io<T>::ld(kr + lane), acc0);
      if (lane + 64 < d) acc1 = fmaf(w, Io<T>::ld(kr + lane + 64), acc1);
    }
    __syncthreads();
  }
  if (lane < d) Io<T>::st(dQ + lane, acc0 * a.scale);
  if (lane + 64 < d) Io<T>::st(dQ + lane + 64, acc1 * a.scale);
}

// dK_j = scale * sum_{h in group} sum_p dS_pj Q_p ; dV_j = sum_h sum_p P_pj dO_p
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_scalar_kernel(AttnArgs a) {
  __shared__ float ks[128];
  __shared__ float vs[128];
  __shared__ float pch[64];
  __shared__ float dsch[64];
  const int j = blockIdx.x, g = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const SeqView sv = seq_view(a, b);
  if (j >= sv.L) return;                               // packed batch: a shorter entry
  const int d = a.d, rep = a.H / a.G;
  const int64_t kvrow = ((sv.kv0 + j) * a.G + g) * d;
  const T* K = (const T*)a.k + kvrow;
  const T* V = (const T*)a.v + kvrow;
  T* dK = (T*)a.dk + kvrow;
  T* dV = (T*)a.dv + kvrow;
  for (int c = lane; c < d; c += 64) { ks[c] = Io<T>::ld(K + c); vs[c] = Io<T>::ld(V + c); }
  __syncthreads();
  const int pstart = first_query_seeing(j, sample_mask(a, b));
  const int64_t qst = (int64_t)a.H * d;
  float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
  for (int hh = 0; hh < rep; ++hh) {
    const int h = g * rep + hh;
    const T* Q = (const T*)a.q + (sv.q0 * a.H + h) * d;
    const T* dO = (const T*)a.dout + (sv.q0 * a.H + h) * d;
    const float* lse = a.lse + sv.lse0 + h * sv.lse_hs;
    const float* dl = a.delta + sv.lse0 + h * sv.lse_hs;
    for (int p0 = pstart; p0 < sv.S; p0 += 64) {
      int p = p0 + lane;
      float pj = 0.f, ds = 0.f;
      if (p < sv.S && j < row_limit(p, sample_mask(a, b))) {
        pj = expf(a.scale * dot_row(ks, Q + p * qst, d) - lse[p]);
        float dp = dot_row(vs, dO + p * qst, d);
        ds = pj * (dp - dl[p]);
      }
      pch[lane] = pj; dsch[lane] = ds;
      __syncthreads();
      int cnt = min(64, sv.S - p0);
      for (int pp = 0; pp < cnt; ++pp) {
        const T* qr = Q + (int64_t)(p0 + pp) * qst;
        const T* dr = dO + (int64_t)(p0 + pp) * qst;
        float w = dsch[pp], u = pch[pp];
        if (lane < d) { dk0 = fmaf(w, Io<T>::ld(qr + lane), dk0); dv0 = fmaf(u, Io<T>::ld(dr + lane), dv0); }
        if (lane + 64 < d) { dk1 = fmaf(w, Io<T>::ld(qr + lane + 64), dk1); dv1 = fmaf(u, Io<T>::ld(dr + lane + 64), dv1); }
      }
      __syncthreads();
    }
  }
  if (lane < d) { Io<T>::st(dK + lane, dk0 * a.scale); Io<T>::st(dV + lane, dv0); }
  if (lane + 64 < d) { Io<T>::st(dK + lane + 64, dk1 * a.scale); Io<T>::st(dV + lane + 64, dv1); }
}

template <typename T>
static void attn_fwd_scalar(const AttnArgs& a, hipStream_t s, const char* name) {
  ProfScope ps(name, s);
  hipLaunchKernelGGL((attn_fwd_scalar_kernel<T>), dim3(a.S, a.H, a.B), dim3(64), 0, s, a);
}
template <typename T>
static void attn_bwd_scalar(const AttnArgs& a, hipStream_t s, const char* n1, const char* n2) {
  {
    ProfScope ps(n1, s);
    hipLaunchKernelGGL((attn_bwd_dq_scalar_kernel<T>), dim3(a.S, a.H, a.B), dim3(64), 0, s, a);
  }
  {
    ProfScope ps(n2, s);
    hipLaunchKernelGGL((attn_bwd_dkv_scalar_kernel<T>), dim3(a.L, a.G, a.B), dim3(64), 0, s, a);
  }
}

void launch_attn_fwd_f32(const AttnArgs& a, hipStream_t s) { attn_fwd_scalar<float>(a, s, "attn_fwd_f32"); }
// --------------------------------------------------------------------------
// Late-stage simulation (section 4.2, second half): every query also sees the
// predicted states of at most t earlier positions of its own window.  That
// band is a handful of keys per query, so it runs as plain FMA code, one
// wavefront per query row (forward, dQ) or per predicted key row (dKp, dVp),
// lanes owning head channels:
//   forward : (O, LSE) of the masked attention over the true keys is merged
//             with the band: LSE' = logaddexp(LSE, lse_band), O' the weighted mean;
//   backward: the main kernels, given LSE' and delta = rowsum(dO * O'), already
//             produce the true-key parts; the band adds its share to dQ and
//             yields dKp, dVp (zero on rows that no query sees).
// --------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void sim_band_fwd_kernel(SimArgs s) {
  const AttnArgs& a = s.a;
  const int p = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const SeqView sv = seq_view(a, b);
  if (p >= sv.S) return;                               // packed batch: a shorter entry
  int lo, hi;
  sim_band(p, a.mask.k, sample_mask(a, b).eps, s.t, sv.L, lo, hi);
  if (hi <= lo) return;
  const int d = a.d, g = h / (a.H / a.G);
  const int64_t kvs = (int64_t)a.G * d;
  const T* Q = (const T*)a.q + ((sv.q0 + p) * a.H + h) * d;
  T* O = (T*)a.o + ((sv.q0 + p) * a.H + h) * d;
  const T* Kp = (const T*)s.kp + (sv.kv0 * a.G + g) * d;
  const T* Vp = (const T*)s.vp + (sv.kv0 * a.G + g) * d;
  const int64_t li = sv.lse0 + h * sv.lse_hs + p;
  const bool c0 = lane < d, c1 = lane + 64 < d;
  const float q0 = c0 ? Io<T>::ld(Q + lane) : 0.f, q1 = c1 ? Io<T>::ld(Q + lane + 64) : 0.f;
  float m = a.lse[li];                                   // weight of the true-key part: exp(m) * 1
  float l = m > -INFINITY ? 1.f : 0.f;
  float acc0 = (c0 && l > 0.f) ? Io<T>::ld(O + lane) : 0.f, acc1 = (c1 && l > 0.f) ? Io<T>::ld(O + lane + 64) : 0.f;
  for (int j = lo; j < hi; ++j) {
    const T* kr = Kp + j * kvs;
    const T* vr = Vp + j * kvs;
    const float sc = a.scale * wave_sum((c0 ? q0 * Io<T>::ld(kr + lane) : 0.f) + (c1 ? q1 * Io<T>::ld(kr + lane + 64) : 0.f));
    const float mn = fmaxf(m, sc);
    const float al = expf(m - mn), pj = expf(sc - mn);   // m = -inf: al = 0
    acc0 = acc0 * al + (c0 ? pj * Io<T>::ld(vr + lane) : 0.f);
    acc1 = acc1 * al + (c1 ? pj * Io<T>::ld(vr + lane + 64) : 0.f);
    l = l * al + pj;
    m = mn;
  }
  const float inv = 1.f / l;
  if (c0) Io<T>::st(O + lane, acc0 * inv);
  if (c1) Io<T>::st(O + lane + 64, acc1 * inv);
  if (lane == 0) a.lse[li] = m + logf(l);
}

template <typename T>
__global__ __launch_bounds__(64) void sim_band_bwd_dq_kernel(SimArgs s) {
  const AttnArgs& a = s.a;
  const int p = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const SeqView sv = seq_view(a, b);
  if (p >= sv.S) return;                               // packed batch: a shorter entry
  int lo, hi;
  sim_band(p, a.mask.k, sample_mask(a, b).eps, s.t, sv.L, lo, hi);
  if (hi <= lo) return;
  const int d = a.d, g = h / (a.H / a.G);
  const int64_t kvs = (int64_t)a.G * d;
  const int64_t row = ((sv.q0 + p) * a.H + h) * d;
  const T* Q = (const T*)a.q + row;
  const T* dO = (const T*)a.dout + row;
  T* dQ = (T*)a.dq + row;
  const T* Kp = (const T*)s.kp + (sv.kv0 * a.G + g) * d;
  const T* Vp = (const T*)s.vp + (sv.kv0 * a.G + g) * d;
  const int64_t li = sv.lse0 + h * sv.lse_hs + p;
  const bool c0 = lane < d, c1 = lane + 64 < d;
  const float q0 = c0 ? Io<T>::ld(Q + lane) : 0.f, q1 = c1 ? Io<T>::ld(Q + lane + 64) : 0.f;
  const float g0 = c0 ? Io<T>::ld(dO + lane) : 0.f, g1 = c1 ? Io<T>::ld(dO + lane + 64) : 0.f;
  const float lse = a.lse[li], delta = a.delta[li];
  float a0 = 0.f, a1 = 0.f;
  for (int j = lo; j < hi; ++j) {
    const T* kr = Kp + j * kvs;
    const T* vr = Vp + j * kvs;
    const float k0 = c0 ? Io<T>::ld(kr + lane) : 0.f, k1 = c1 ? Io<T>::ld(kr + lane + 64) : 0.f;
    const float v0 = c0 ? Io<T>::ld(vr + lane) : 0.f, v1 = c1 ? Io<T>::ld(vr + lane + 64) : 0.f;
    const float pj = expf(a.scale * wave_sum(q0 * k0 + q1 * k1) - lse);
    const float ds = pj * (wave_sum(g0 * v0 + g1 * v1) - delta);
    a0 = fmaf(ds, k0, a0);
    a1 = fmaf(ds, k1, a1);
  }
  if (c0) Io<T>::st(dQ + lane, Io<T>::ld(dQ + lane) + a0 * a.scale);
  if (c1) Io<T>::st(dQ + lane + 64, Io<T>::ld(dQ + lane + 64) + a1 * a.scale);
}

template <typename T>
__global__ __launch_bounds__(64) void sim_band_bwd_dkv_kernel(SimArgs s) {
  const AttnArgs& a = s.a;
  const int j = blockIdx.x, g = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const SeqView sv = seq_view(a, b);
  if (j >= sv.L) return;                               // packed batch: a shorter entry
  const int d = a.d, rep = a.H / a.G;
  const int64_t kvrow = ((sv.kv0 + j) * a.G + g) * d;
  const T* kr = (const T*)s.kp + kvrow;
  const T* vr = (const T*)s.vp + kvrow;
  const bool c0 = lane < d, c1 = lane + 64 < d;
  float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
  const int w0 = window_start_raw(j, a.mask.k, sample_mask(a, b).eps);
  if (j - w0 < s.t) {                                  // this position holds a predicted state at step t
    const float k0 = c0 ? Io<T>::ld(kr + lane) : 0.f, k1 = c1 ? Io<T>::ld(kr + lane + 64) : 0.f;
    const float v0 = c0 ? Io<T>::ld(vr + lane) : 0.f, v1 = c1 ? Io<T>::ld(vr + lane + 64) : 0.f;
    const int p_end = min(w0 + a.mask.k, sv.S);         // the later queries of the same window see it
    for (int p = j + 1; p < p_end; ++p)
      for (int hh = 0; hh < rep; ++hh) {
        const int h = g * rep + hh;
        const int64_t row = ((sv.q0 + p) * a.H + h) * d;
        const T* Q = (const T*)a.q + row;
        const T* dO = (const T*)a.dout + row;
        const int64_t li = sv.lse0 + h * sv.lse_hs + p;
        const float q0 = c0 ? Io<T>::ld(Q + lane) : 0.f, q1 = c1 ? Io<T>::ld(Q + lane + 64) : 0.f;
        const float g0 = c0 ? Io<T>::ld(dO + lane) : 0.f, g1 = c1 ? Io<T>::ld(dO + lane + 64) : 0.f;
        const float pj = expf(a.scale * wave_sum(q0 * k0 + q1 * k1) - a.lse[li]);
        const float ds = pj * (wave_sum(g0 * v0 + g1 * v1) - a.delta[li]);
        dk0 = fmaf(ds, q0, dk0); dk1 = fmaf(ds, q1, dk1);
        dv0 = fmaf(pj, g0, dv0); dv1 = fmaf(pj, g1, dv1);
      }
  }
  T* dK = (T*)s.dkp + kvrow;
  T* dV = (T*)s.dvp + kvrow;
  if (c0) { Io<T>::st(dK + lane, dk0 * a.scale); Io<T>::st(dV + lane, dv0); }
  if (c1) { Io<T>::st(dK + lane + 64, dk1 * a.scale); Io<T>::st(dV + lane + 64, dv1); }
}

void launch_sim_band_fwd(const SimArgs& s, hipStream_t st) {
  if (s.is_bf16) return launch_sim_band_fwd_bf16(s, st);    // bf16 storage implies head width 128
  ProfScope ps("sim_band_fwd", st);
  dim3 grid(s.a.S, s.a.H, s.a.B);
  hipLaunchKernelGGL(sim_band_fwd_kernel<float>, grid, dim3(64), 0, st, s);
}
void launch_sim_band_bwd(const SimArgs& s, hipStream_t st) {
  if (s.is_bf16) return launch_sim_band_bwd_bf16(s, st);
  {
    ProfScope ps("sim_band_bwd_dq", st);
    dim3 grid(s.a.S, s.a.H, s.a.B);
    hipLaunchKernelGGL(sim_band_bwd_dq_kernel<float>, grid, dim3(64), 0, st, s);
  }
  {
    ProfScope ps("sim_band_bwd_dkv", st);
    dim3 grid(s.a.L, s.a.G, s.a.B);
    hipLaunchKernelGGL(sim_band_bwd_dkv_kernel<float>, grid, dim3(64), 0, st, s);
  }
}

// In-place update of the predicted-state buffer between simulation steps (section 4.2, second half):
// after step t the row at position t of every window takes the newly predicted state of that position.
// blockIdx.x: window (the partial leading one first), blockIdx.y: batch entry; rows as 16-byte chunks.
__global__ __launch_bounds__(256) void sim_save_kernel(const uint4* __restrict__ h, uint4* __restrict__ xpred, int L,
                                                       int chunks, int k, int eps, const int32_t* eps_b, int t,
                                                       const int32_t* cu, int total) {
  if (eps_b) { eps = eps_b[blockIdx.y] % k; if (eps < 0) eps += k; }
  int64_t first = (int64_t)blockIdx.y * L;          // first row of this entry
  if (cu) {                                          // packed batch: clamped like the attention kernels' view
    const int32_t r0 = min(max(cu[blockIdx.y], 0), total);
    L = min(max(cu[blockIdx.y + 1] - r0, 0), min(L, total - r0));
    first = r0;
  }
  const int n0 = eps > 0 ? eps - k : 0;
  const int j = n0 + (int)blockIdx.x * k + t;
  if (j < 0 || j >= L) return;
  const int64_t row = (first + j) * chunks;
  for (int c = threadIdx.x; c < chunks; c += 256) xpred[row + c] = h[row + c];
}

void launch_sim_save(const void* h, void* xpred, int B, int L, int64_t row_bytes, int k, int eps, const int32_t* eps_b,
                     int t, const int32_t* cu, int total, hipStream_t st) {
  ProfScope ps("sim_save", st);
  const int n0 = (eps_b || eps > 0) ? -k + 1 : 0;   // lowest possible start of the leading window
  const int n_win = (L - n0 + k - 1) / k + 1;
  hipLaunchKernelGGL(sim_save_kernel, dim3(n_win, B), dim3(256), 0, st, (const uint4*)h, (uint4*)xpred, L,
                     (int)(row_bytes / 16), k, eps, eps_b, t, cu, total);
}

void launch_attn_bwd_f32(const AttnArgs& a, hipStream_t s) {
  attn_bwd_scalar<float>(a, s, "attn_bwd_dq_f32", "attn_bwd_dkv_f32");
}

}  // namespace beagle
