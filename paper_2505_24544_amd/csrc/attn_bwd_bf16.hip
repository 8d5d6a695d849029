// Backward of the block-masked cross-attention for bf16, head width 128, on
// gfx950 MFMA, by recomputation from Q, K, V, O, dO and the stored LSE:
//   delta_p = sum_c dO_pc O_pc          P = exp(s - LSE)        dS = P * (dP - delta)
//   dQ = scale * dS K      dK = scale * dS^T Q      dV = P^T dO      dP = dO V^T
//
// Two kernels, no floating-point atomics (results are bitwise reproducible):
//
//  (1) dq kernel   one workgroup = 128 queries of one (b, h), loop over the key
//      tiles those queries can see.  As in the forward, a lane owns ONE query:
//      S^T = K Q^T and dP^T = V dO^T come out with column q = lane % 32, so LSE
//      and delta are per-lane scalars, and dS^T goes straight from the
//      accumulator registers into the B operand of dQ^T += K^T dS^T.  The kernel
//      also computes delta and stores it for kernel (2).
//
//  (2) dkv kernel  one workgroup = 128 keys of one (b, kv head), loop over the
//      H/G query heads of the group and over the query tiles that can see those
//      keys.  A lane owns ONE key: S = Q K^T and dP = dO V^T come out with
//      column j = lane % 32; P and dS go straight into the B operands of
//      dV^T += dO^T P and dK^T += Q^T dS.  LSE/delta of the tile's queries are
//      read from LDS (they index the accumulator registers here).
//
// LDS tiles hold rows of 128 channels (256 B) in HBM order with the 16-byte
// chunks of row r XOR-swizzled by ((r & 3) << 2 | (r >> 2) & 3).  That makes
// both access patterns bank-conflict free on the same tile: whole-row
// ds_read_b128 fragments (k = channel) and ds_read_b64_tr_b16 transpose
// fragments (k = row).
//
// Mask: query p sees key j iff j < row_limit(p) iff p >= first_query_seeing(j).
// Key tiles beyond a workgroup's last limit / query tiles before a key tile's
// first viewer are never visited (whole-tile skipping).
#include "common.h"

namespace beagle {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4_t;
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;

namespace bwd {
constexpr int HD = 128;
constexpr int ROW = HD;                 // elements per LDS row (no padding; swizzled)
constexpr float LOG2E = 1.44269504088896340736f;

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// whole-row fragment: row r, channels 16 s + 8 hf .. + 7
__device__ __forceinline__ bf16x8_t row_frag(const bf16_t* tile, int r, int s, int hf) {
  return *(const bf16x8_t*)(tile + r * ROW + (((2 * s + hf) ^ swz(r)) << 3));
}

// transpose fragment: lane gets rows rowbase + {4 hf + 0..3, 8 + 4 hf + 0..3} of channel 32 cb + lane % 32
__device__ __forceinline__ bf16x8_t tr_frag(const bf16_t* tile, int rowbase, int cb, int lane) {
  const int gi = lane >> 4, r = lane & 15;
  const int row = rowbase + 4 * (gi >> 1) + (r >> 2);
  const int chunk = 4 * cb + 2 * (gi & 1) + ((r & 3) >> 1);
  const int sub = 4 * (r & 1);
  const bf16_t* p0 = tile + row * ROW + ((chunk ^ swz(row)) << 3) + sub;
  const bf16_t* p1 = tile + (row + 8) * ROW + ((chunk ^ swz(row + 8)) << 3) + sub;
  union { struct { s16x4_t x, y; } s; bf16x8_t v; } f;
  f.s.x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
  f.s.y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p1);
  return f.v;
}

__device__ __forceinline__ void store_chunk(bf16_t* tile, int r, int chunk, i32x4_t v) {
  *(i32x4_t*)(tile + r * ROW + ((chunk ^ swz(r)) << 3)) = v;
}

__device__ __forceinline__ uint32_t cvt_pk(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return *(uint32_t*)&b;
}
__device__ __forceinline__ float dot8(bf16x8_t a, bf16x8_t b) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s = fmaf((float)a[i], (float)b[i], s);
  return s;
}
}  // namespace bwd

// ===========================================================================
// (1) dQ and delta
// ===========================================================================
namespace dqk {
constexpr int BQ = 128, BJ = 64;
constexpr int TILE = BJ * bwd::ROW;            // one K or V tile
constexpr int STAGE = 2 * TILE;
constexpr int CHUNKS = BJ * bwd::HD / 8 / 256;
}  // namespace dqk

__global__ __launch_bounds__(256, 2) void attn_bwd_dq_bf16_kernel(AttnArgs a) {
  using namespace bwd;
  using namespace dqk;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, ql = lane & 31;
  const int nqt = (a.S + BQ - 1) / BQ;
  const int qt = nqt - 1 - blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z, g = h / (a.H / a.G);
  const int q0 = qt * BQ, qw0 = q0 + wave * 32, q = qw0 + ql;
  const bool q_ok = q < a.S;
  const int qc = q_ok ? q : a.S - 1;
  const int64_t qrow = (((int64_t)b * a.S + qc) * a.H + h) * HD;
  const bf16_t* Qg = (const bf16_t*)a.q + qrow;
  const bf16_t* Og = (const bf16_t*)a.o + qrow;
  const bf16_t* dOg = (const bf16_t*)a.dout + qrow;
  const bf16_t* Kg = (const bf16_t*)a.k + ((int64_t)b * a.L * a.G + g) * HD;
  const bf16_t* Vg = (const bf16_t*)a.v + ((int64_t)b * a.L * a.G + g) * HD;
  const int64_t kvs = (int64_t)a.G * HD;
  const int64_t li = ((int64_t)b * a.H + h) * a.S + qc;

  const int lim = q_ok ? row_limit(q, a.mask) : 0;
  const int wg_lim = row_limit(min(q0 + BQ, a.S) - 1, a.mask);
  const int wave_hi = qw0 < a.S ? row_limit(min(qw0 + 32, a.S) - 1, a.mask) : 0;
  const int wave_lo = qw0 < a.S ? row_limit(qw0, a.mask) : 0;
  const int ntiles = (wg_lim + BJ - 1) / BJ;

  bf16x8_t qf[8], dof[8];
  float part = 0.f;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    qf[s] = *(const bf16x8_t*)(Qg + 16 * s + 8 * hf);
    dof[s] = *(const bf16x8_t*)(dOg + 16 * s + 8 * hf);
    bf16x8_t of = *(const bf16x8_t*)(Og + 16 * s + 8 * hf);
    part += dot8(dof[s], of);
  }
  const float delta = part + __shfl_xor(part, 32, 64);
  if (q_ok && hf == 0) a.delta[li] = delta;
  const float lse = a.lse[li];
  const float c2 = a.scale * LOG2E;
  const float lse2 = (lim > 0 ? lse : 0.f) * LOG2E;    // blind rows are fully masked below

  f32x16_t dq[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;

  i32x4_t kr[CHUNKS], vr[CHUNKS];
  auto load_tile = [&](int jt) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = tid + 256 * i, r = c >> 4, ch = c & 15;
      const int j = jt * BJ + r;
      i32x4_t z = {0, 0, 0, 0};
      kr[i] = z; vr[i] = z;
      if (j < a.L) {
        kr[i] = *(const i32x4_t*)(Kg + j * kvs + ch * 8);
        vr[i] = *(const i32x4_t*)(Vg + j * kvs + ch * 8);
      }
    }
  };
  auto store_tile = [&](int stage) {
    bf16_t* ks = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = tid + 256 * i, r = c >> 4, ch = c & 15;
      store_chunk(ks, r, ch, kr[i]);
      store_chunk(ks + TILE, r, ch, vr[i]);
    }
  };
  if (ntiles > 0) { load_tile(0); store_tile(0); }
  __syncthreads();

#pragma unroll 1
  for (int jt = 0; jt < ntiles; ++jt) {
    const int cur = jt & 1;
    const bool more = jt + 1 < ntiles;
    if (more) load_tile(jt + 1);
    const int j0 = jt * BJ;
    if (j0 < wave_hi) {
      const bf16_t* ks = smem + cur * STAGE;
      const bf16_t* vs = ks + TILE;
      f32x16_t st[2], dp[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) { st[jb][e] = 0.f; dp[jb][e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(ks, jb * 32 + ql, s, hf), qf[s], st[jb], 0, 0, 0);
          dp[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(vs, jb * 32 + ql, s, hf), dof[s], dp[jb], 0, 0, 0);
        }
      }
      const bool partial = j0 + BJ > wave_lo;
      uint32_t pk[2][8];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          float ds[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int j = j0 + 32 * jb + 8 * ((e + u) >> 2) + 4 * hf + ((e + u) & 3);
            const float p = __builtin_amdgcn_exp2f(st[jb][e + u] * c2 - lse2);
            const float v = p * (dp[jb][e + u] - delta);
            ds[u] = (partial && j >= lim) ? 0.f : v;
          }
          pk[jb][e >> 1] = cvt_pk(ds[0], ds[1]);
        }
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          union { uint32_t u[4]; bf16x8_t v; } sf;
#pragma unroll
          for (int i = 0; i < 4; ++i) sf.u[i] = pk[jb][4 * t + i];
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            dq[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(ks, 32 * jb + 16 * t, cb, lane), sf.v, dq[cb], 0, 0, 0);
        }
    }
    if (more) store_tile(cur ^ 1);
    __syncthreads();
  }

  if (q_ok) {
    bf16_t* dQg = (bf16_t*)a.dq + qrow;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        uint2 v = {cvt_pk(dq[cb][4 * qd] * a.scale, dq[cb][4 * qd + 1] * a.scale),
                   cvt_pk(dq[cb][4 * qd + 2] * a.scale, dq[cb][4 * qd + 3] * a.scale)};
        *(uint2*)(dQg + 32 * cb + 8 * qd + 4 * hf) = v;
      }
  }
}

// ===========================================================================
// (2) dK and dV
// ===========================================================================
namespace dkv {
constexpr int BJ = 128, BQ = 64;
constexpr int TILE = BQ * bwd::ROW;            // one Q or dO tile
constexpr int STAGE = 2 * TILE;
constexpr int CHUNKS = BQ * bwd::HD / 8 / 256;
constexpr int STAT_OFF = 2 * STAGE;            // in bf16 elements; floats follow: [stage][lse 64 | delta 64]
}  // namespace dkv

__global__ __launch_bounds__(256, 1) void attn_bwd_dkv_bf16_kernel(AttnArgs a) {
  using namespace bwd;
  using namespace dkv;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  float* stat = (float*)(smem + STAT_OFF);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, jl = lane & 31;
  const int jt = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int rep = a.H / a.G;
  const int j0 = jt * BJ, jw0 = j0 + wave * 32, j = jw0 + jl;
  const bool j_ok = j < a.L;
  const int jc = j_ok ? j : a.L - 1;
  const int64_t kvrow = (((int64_t)b * a.L + jc) * a.G + g) * HD;
  const bf16_t* Kg = (const bf16_t*)a.k + kvrow;
  const bf16_t* Vg = (const bf16_t*)a.v + kvrow;
  const int64_t qs = (int64_t)a.H * HD;

  // first query that sees this lane's key / any key of the wave / every key of the wave / any of the workgroup
  const int fq = j_ok ? first_query_seeing(j, a.mask) : a.S;
  const int wave_first = jw0 < a.L ? first_query_seeing(jw0, a.mask) : a.S;
  const int wave_all = jw0 < a.L ? first_query_seeing(min(jw0 + 32, a.L) - 1, a.mask) : a.S;
  const int wg_first = first_query_seeing(j0, a.mask);
  const int qt0 = wg_first / BQ;
  const int nqt = (a.S + BQ - 1) / BQ;

  bf16x8_t kf[8], vf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    kf[s] = *(const bf16x8_t*)(Kg + 16 * s + 8 * hf);
    vf[s] = *(const bf16x8_t*)(Vg + 16 * s + 8 * hf);
  }
  const float c2 = a.scale * LOG2E;

  f32x16_t dk[4], dv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[i][e] = 0.f; dv[i][e] = 0.f; }

  const int iters = (nqt > qt0 ? nqt - qt0 : 0) * rep;    // (head, query tile) pairs, head-major
  i32x4_t qr[CHUNKS], dr[CHUNKS];
  float st_l = 0.f, st_d = 0.f;
  auto coords = [&](int it, int& h, int& q0) { h = g * rep + it / (nqt - qt0); q0 = (qt0 + it % (nqt - qt0)) * BQ; };
  auto load_tile = [&](int it) {
    int h, q0; coords(it, h, q0);
    const bf16_t* Qg = (const bf16_t*)a.q + ((int64_t)b * a.S * a.H + h) * HD;
    const bf16_t* dOg = (const bf16_t*)a.dout + ((int64_t)b * a.S * a.H + h) * HD;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = tid + 256 * i, r = c >> 4, ch = c & 15;
      const int p = q0 + r;
      i32x4_t z = {0, 0, 0, 0};
      qr[i] = z; dr[i] = z;
      if (p < a.S) {
        qr[i] = *(const i32x4_t*)(Qg + p * qs + ch * 8);
        dr[i] = *(const i32x4_t*)(dOg + p * qs + ch * 8);
      }
    }
    if (tid < BQ) {
      const int p = q0 + tid;
      const int64_t li = ((int64_t)b * a.H + h) * a.S + p;
      // padding rows: LSE = +inf makes their probabilities exactly zero
      st_l = p < a.S ? a.lse[li] * LOG2E : INFINITY;
      st_d = p < a.S ? a.delta[li] : 0.f;
    }
  };
  auto store_tile = [&](int stage) {
    bf16_t* qsm = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = tid + 256 * i, r = c >> 4, ch = c & 15;
      store_chunk(qsm, r, ch, qr[i]);
      store_chunk(qsm + TILE, r, ch, dr[i]);
    }
    if (tid < BQ) { stat[stage * 128 + tid] = st_l; stat[stage * 128 + 64 + tid] = st_d; }
  };
  if (iters > 0) { load_tile(0); store_tile(0); }
  __syncthreads();

#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
    const int cur = it & 1;
    const bool more = it + 1 < iters;
    if (more) load_tile(it + 1);
    int h, q0; coords(it, h, q0);
    if (q0 + BQ > wave_first) {                       // some query of the tile sees some key of the wave
      const bf16_t* qsm = smem + cur * STAGE;
      const bf16_t* dsm = qsm + TILE;
      const float* sl = stat + cur * 128;
      f32x16_t s2[2], dp[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) { s2[qb][e] = 0.f; dp[qb][e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          s2[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(qsm, qb * 32 + jl, s, hf), kf[s], s2[qb], 0, 0, 0);
          dp[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(dsm, qb * 32 + jl, s, hf), vf[s], dp[qb], 0, 0, 0);
        }
      }
      // register e of block qb is query q0 + 32 qb + 8 (e/4) + 4 hf + e%4 ; column = this lane's key
      const bool partial = q0 < wave_all;
      uint32_t pp[2][8], pd[2][8];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int r = 32 * qb + 8 * e4 + 4 * hf;
          const float4 l4 = *(const float4*)(sl + r);
          const float4 d4 = *(const float4*)(sl + 64 + r);
          const float ls[4] = {l4.x, l4.y, l4.z, l4.w};
          const float dl[4] = {d4.x, d4.y, d4.z, d4.w};
          float pv[4], dsv[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = 4 * e4 + u;
            float p = __builtin_amdgcn_exp2f(s2[qb][e] * c2 - ls[u]);
            if (partial && q0 + r + u < fq) p = 0.f;
            pv[u] = p;
            dsv[u] = p * (dp[qb][e] - dl[u]);
          }
          pp[qb][2 * e4] = cvt_pk(pv[0], pv[1]); pp[qb][2 * e4 + 1] = cvt_pk(pv[2], pv[3]);
          pd[qb][2 * e4] = cvt_pk(dsv[0], dsv[1]); pd[qb][2 * e4 + 1] = cvt_pk(dsv[2], dsv[3]);
        }
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          union { uint32_t u[4]; bf16x8_t v; } pf, sf;
#pragma unroll
          for (int i = 0; i < 4; ++i) { pf.u[i] = pp[qb][4 * t + i]; sf.u[i] = pd[qb][4 * t + i]; }
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) {
            dv[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(dsm, 32 * qb + 16 * t, cb, lane), pf.v, dv[cb], 0, 0, 0);
            dk[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(qsm, 32 * qb + 16 * t, cb, lane), sf.v, dk[cb], 0, 0, 0);
          }
        }
    }
    if (more) store_tile(cur ^ 1);
    __syncthreads();
  }

  if (j_ok) {
    bf16_t* dKg = (bf16_t*)a.dk + kvrow;
    bf16_t* dVg = (bf16_t*)a.dv + kvrow;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        uint2 v = {cvt_pk(dk[cb][4 * qd] * a.scale, dk[cb][4 * qd + 1] * a.scale),
                   cvt_pk(dk[cb][4 * qd + 2] * a.scale, dk[cb][4 * qd + 3] * a.scale)};
        uint2 w = {cvt_pk(dv[cb][4 * qd], dv[cb][4 * qd + 1]), cvt_pk(dv[cb][4 * qd + 2], dv[cb][4 * qd + 3])};
        *(uint2*)(dKg + 32 * cb + 8 * qd + 4 * hf) = v;
        *(uint2*)(dVg + 32 * cb + 8 * qd + 4 * hf) = w;
      }
  }
}

size_t attn_bwd_bf16_ws_bytes(const AttnArgs&) { return 0; }

void launch_attn_bwd_bf16(const AttnArgs& a, void*, hipStream_t s) {
  {
    constexpr size_t smem = 2 * (size_t)dqk::STAGE * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
      (void)hipFuncSetAttribute((const void*)attn_bwd_dq_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      attr_set = true;
    }
    ProfScope ps("attn_bwd_dq_bf16", s);
    dim3 grid((a.S + dqk::BQ - 1) / dqk::BQ, a.H, a.B);
    hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel, grid, dim3(256), smem, s, a);
  }
  {
    constexpr size_t smem = 2 * (size_t)dkv::STAGE * sizeof(bf16_t) + 2 * 128 * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
      (void)hipFuncSetAttribute((const void*)attn_bwd_dkv_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      attr_set = true;
    }
    ProfScope ps("attn_bwd_dkv_bf16", s);
    dim3 grid((a.L + dkv::BJ - 1) / dkv::BJ, a.G, a.B);
    hipLaunchKernelGGL(attn_bwd_dkv_bf16_kernel, grid, dim3(256), smem, s, a);
  }
}

}  // namespace beagle
