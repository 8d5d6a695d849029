// Late-stage simulation band (section 4.2, second half) for bf16 storage and
// head width 128.  Same arithmetic as the one-wave-per-row kernels of the
// scalar path, laid out for memory throughput: the band is at most t keys per
// query, so these kernels are pure streaming over Q / O / dO / dQ.  A row of 128
// channels is owned by 16 lanes with one 16-byte chunk each (a wavefront covers
// four consecutive rows = 1 KB contiguous), dot products are reduced inside a
// 16-lane DPP row, and no LDS is used.
//   grid.x: blocks of 16 rows of one batch element, grid.y: batch elements.
#include "common.h"
#include "mask_index.h"

namespace beagle {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int BD = 128;          // head width
constexpr int ROWS_PER_WG = 16;  // 256 threads / 16 lanes per row

// Sum over the 16 lanes of a DPP row; every lane gets the total.
__device__ __forceinline__ float row16_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));  // row_half_mirror
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true));  // row_mirror
  return v;
}

struct Chunk { float f[8]; };

__device__ __forceinline__ Chunk load_chunk(const bf16_t* row, int c) {
  const u32x4 w = *(const u32x4*)(row + 8 * c);
  Chunk x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x.f[2 * i] = __uint_as_float(w[i] << 16);
    x.f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
  return x;
}

__device__ __forceinline__ void store_chunk(bf16_t* row, int c, const Chunk& x) {
  u32x4 w;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = (uint32_t)f32_to_bf16(x.f[2 * i]) | ((uint32_t)f32_to_bf16(x.f[2 * i + 1]) << 16);
  *(u32x4*)(row + 8 * c) = w;
}

__device__ __forceinline__ float dot8(const Chunk& a, const Chunk& b) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s = fmaf(a.f[i], b.f[i], s);
  return s;
}

// Forward: merge the band into (O, LSE) of the masked attention over the true keys.
__global__ __launch_bounds__(256) void sim_band_fwd_bf16_kernel(SimArgs s) {
  const AttnArgs& a = s.a;
  const int rb = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (rb >= a.S * a.H) return;
  const int p = rb / a.H, h = rb - p * a.H, g = h / (a.H / a.G);
  for (int b = blockIdx.y; b < a.B; b += gridDim.y) {
    const SeqView sv = seq_view(a, b);
    if (p >= sv.S) continue;                               // packed batch: a shorter entry
    int lo, hi;
    sim_band(p, a.mask.k, sample_mask(a, b).eps, s.t, sv.L, lo, hi);
    if (hi <= lo) continue;
    const int64_t row = (sv.q0 * a.H + rb) * BD;
    const bf16_t* Kp = (const bf16_t*)s.kp + (sv.kv0 * a.G + g) * BD;
    const bf16_t* Vp = (const bf16_t*)s.vp + (sv.kv0 * a.G + g) * BD;
    const int64_t li = sv.lse0 + h * sv.lse_hs + p;
    const Chunk q = load_chunk((const bf16_t*)a.q + row, c);
    float m = a.lse[li];                                   // weight of the true-key part: exp(m) * 1
    float l = m > -INFINITY ? 1.f : 0.f;
    Chunk acc = load_chunk((const bf16_t*)a.o + row, c);
    if (l == 0.f)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc.f[i] = 0.f;
    for (int j = lo; j < hi; ++j) {
      const Chunk kk = load_chunk(Kp + (int64_t)j * a.G * BD, c);
      const Chunk vv = load_chunk(Vp + (int64_t)j * a.G * BD, c);
      const float sc = a.scale * row16_sum(dot8(q, kk));
      const float mn = fmaxf(m, sc);
      const float al = expf(m - mn), pj = expf(sc - mn);   // m = -inf: al = 0
#pragma unroll
      for (int i = 0; i < 8; ++i) acc.f[i] = fmaf(pj, vv.f[i], acc.f[i] * al);
      l = fmaf(l, al, pj);
      m = mn;
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc.f[i] *= inv;
    store_chunk((bf16_t*)a.o + row, c, acc);
    if (c == 0) a.lse[li] = m + logf(l);
  }
}

// dQ += scale * sum_j dS_j Kp_j over the band.
__global__ __launch_bounds__(256) void sim_band_bwd_dq_bf16_kernel(SimArgs s) {
  const AttnArgs& a = s.a;
  const int rb = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (rb >= a.S * a.H) return;
  const int p = rb / a.H, h = rb - p * a.H, g = h / (a.H / a.G);
  for (int b = blockIdx.y; b < a.B; b += gridDim.y) {
    const SeqView sv = seq_view(a, b);
    if (p >= sv.S) continue;                               // packed batch: a shorter entry
    int lo, hi;
    sim_band(p, a.mask.k, sample_mask(a, b).eps, s.t, sv.L, lo, hi);
    if (hi <= lo) continue;
    const int64_t row = (sv.q0 * a.H + rb) * BD;
    const bf16_t* Kp = (const bf16_t*)s.kp + (sv.kv0 * a.G + g) * BD;
    const bf16_t* Vp = (const bf16_t*)s.vp + (sv.kv0 * a.G + g) * BD;
    const int64_t li = sv.lse0 + h * sv.lse_hs + p;
    const Chunk q = load_chunk((const bf16_t*)a.q + row, c);
    const Chunk go = load_chunk((const bf16_t*)a.dout + row, c);
    Chunk dq = load_chunk((const bf16_t*)a.dq + row, c);
    const float lse = a.lse[li], delta = a.delta[li];
    Chunk acc;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc.f[i] = 0.f;
    for (int j = lo; j < hi; ++j) {
      const Chunk kk = load_chunk(Kp + (int64_t)j * a.G * BD, c);
      const Chunk vv = load_chunk(Vp + (int64_t)j * a.G * BD, c);
      const float pj = expf(a.scale * row16_sum(dot8(q, kk)) - lse);
      const float ds = pj * (row16_sum(dot8(go, vv)) - delta);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc.f[i] = fmaf(ds, kk.f[i], acc.f[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) dq.f[i] += acc.f[i] * a.scale;
    store_chunk((bf16_t*)a.dq + row, c, dq);
  }
}

// dKp, dVp of every predicted key row (zeros on rows that no query sees).
__global__ __launch_bounds__(256) void sim_band_bwd_dkv_bf16_kernel(SimArgs s) {
  const AttnArgs& a = s.a;
  const int rb = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (rb >= a.L * a.G) return;
  const int j = rb / a.G, g = rb - j * a.G, rep = a.H / a.G;
  for (int b = blockIdx.y; b < a.B; b += gridDim.y) {
    const SeqView sv = seq_view(a, b);
    if (j >= sv.L) continue;                               // packed batch: a shorter entry
    const int w0 = window_start_raw(j, a.mask.k, sample_mask(a, b).eps);
    const bool holds_pred = j - w0 < s.t;                  // this position holds a predicted state at step t
    const int p_end = min(w0 + a.mask.k, sv.S);            // the later queries of the same window see it
    const int64_t kvrow = (sv.kv0 * a.G + rb) * BD;
    Chunk dk, dv;
#pragma unroll
    for (int i = 0; i < 8; ++i) dk.f[i] = dv.f[i] = 0.f;
    if (holds_pred) {
      const Chunk kk = load_chunk((const bf16_t*)s.kp + kvrow, c);
      const Chunk vv = load_chunk((const bf16_t*)s.vp + kvrow, c);
      for (int p = j + 1; p < p_end; ++p)
        for (int hh = 0; hh < rep; ++hh) {
          const int h = g * rep + hh;
          const int64_t row = ((sv.q0 + p) * a.H + h) * BD;
          const int64_t li = sv.lse0 + h * sv.lse_hs + p;
          const Chunk q = load_chunk((const bf16_t*)a.q + row, c);
          const Chunk go = load_chunk((const bf16_t*)a.dout + row, c);
          const float pj = expf(a.scale * row16_sum(dot8(q, kk)) - a.lse[li]);
          const float ds = pj * (row16_sum(dot8(go, vv)) - a.delta[li]);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            dk.f[i] = fmaf(ds, q.f[i], dk.f[i]);
            dv.f[i] = fmaf(pj, go.f[i], dv.f[i]);
          }
        }
#pragma unroll
      for (int i = 0; i < 8; ++i) dk.f[i] *= a.scale;
    }
    store_chunk((bf16_t*)s.dkp + kvrow, c, dk);
    store_chunk((bf16_t*)s.dvp + kvrow, c, dv);
  }
}

dim3 band_grid(int rows_per_batch, int B) {
  return dim3((rows_per_batch + ROWS_PER_WG - 1) / ROWS_PER_WG, B < 65535 ? B : 65535);
}

}  // namespace

void launch_sim_band_fwd_bf16(const SimArgs& s, hipStream_t st) {
  ProfScope ps("sim_band_fwd_bf16", st);
  hipLaunchKernelGGL(sim_band_fwd_bf16_kernel, band_grid(s.a.S * s.a.H, s.a.B), dim3(256), 0, st, s);
}

void launch_sim_band_bwd_bf16(const SimArgs& s, hipStream_t st) {
  {
    ProfScope ps("sim_band_bwd_dq_bf16", st);
    hipLaunchKernelGGL(sim_band_bwd_dq_bf16_kernel, band_grid(s.a.S * s.a.H, s.a.B), dim3(256), 0, st, s);
  }
  {
    ProfScope ps("sim_band_bwd_dkv_bf16", st);
    hipLaunchKernelGGL(sim_band_bwd_dkv_bf16_kernel, band_grid(s.a.L * s.a.G, s.a.B), dim3(256), 0, st, s);
  }
}

}  // namespace beagle
