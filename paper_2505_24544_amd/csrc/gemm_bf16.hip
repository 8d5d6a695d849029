// bf16 GEMM on the gfx950 matrix cores: C[M,N] = X * W (+ X2 * W2), float
// accumulation, for the Q/K/V/output projections of Eq. 2 and every
// projection-shaped contraction of the backward pass.
//
// Design
//   * One workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile of C; each
//     wave owns (32*TM) x (32*TN) of it as TM x TN accumulators of the
//     v_mfma_f32_32x32x16_bf16 instruction.
//   * The k loop walks BK = 64 at a time through two LDS stages: the global
//     loads of slice t+1 are issued before the MFMAs of slice t and parked in
//     registers, then written to the other stage; one barrier per slice.
//   * Each operand tile sits in LDS in the order it has in HBM, so the copy is
//     16 bytes per lane, coalesced, whatever the storage order:
//       k-contiguous operand  -> tile [rows][BK + 8]; a fragment is one
//                                ds_read_b128 (rows padded to 144 B: the 16
//                                lanes of a read phase hit 64 distinct banks);
//       row-contiguous operand-> tile [BK][rows + 32]; a fragment is two
//                                ds_read_b64_tr_b16 (the LDS transpose read),
//                                which hand every lane four consecutive k of
//                                its own row.
//   * The MFMA is issued "transposed" (A operand = W rows, B operand = X rows)
//     so that a lane ends up with 4 consecutive n of one C row in 4 consecutive
//     accumulator registers: the epilogue stores 8 (bf16) or 16 (float) bytes
//     per lane per instruction.
//   * Workgroup ids are remapped so that each XCD (ids are dealt round-robin
//     to the 8 XCDs) works on a contiguous run of tiles, and tiles are walked
//     in groups of GROUP_M tile-rows so that the run shares X and W tiles in
//     that XCD's L2.
//   * Several independent GEMMs can share one launch (Q, K, V projections;
//     the three weight gradients) so that small ones do not leave CUs idle.
#include "common.h"

namespace beagle {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4_t;

constexpr int BK = 64;
constexpr int KPAD = 8;     // k-contiguous tiles: row stride BK + 8 elements
constexpr int RPAD = 32;    // row-contiguous tiles: k-row stride rows + 32 elements
constexpr int GROUP_M = 4;
constexpr int NUM_XCD = 8;

template <int ROWS, bool KMAJOR>
struct TileGeom {
  static constexpr int LD = KMAJOR ? (BK + KPAD) : (ROWS + RPAD);
  static constexpr int ELEMS = KMAJOR ? ROWS * LD : BK * LD;
  static constexpr int CHUNKS = ROWS * BK / 8;          // 16-byte chunks per slice
  static constexpr int PER_THREAD = CHUNKS / 256;
};

// Global -> registers for one BK slice of one operand.
//   KMAJOR : element (row r, k) at base[r * ld + k]
//   !KMAJOR: element (row r, k) at base[k * ld + r]
// rows beyond `rows_valid` and k beyond `k_valid` read as zero.
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ void load_slice(i32x4_t* __restrict__ reg,
                                           const bf16_t* __restrict__ base, int64_t ld, int row0, int k0,
                                           int rows_valid, int k_valid, int tid) {
  using G = TileGeom<ROWS, KMAJOR>;
#pragma unroll
  for (int i = 0; i < G::PER_THREAD; ++i) {
    const int c = tid + 256 * i;
    int r, k;
    if (KMAJOR) { r = c / (BK / 8); k = (c % (BK / 8)) * 8; }
    else        { k = c / (ROWS / 8); r = (c % (ROWS / 8)) * 8; }
    const int gr = row0 + r, gk = k0 + k;
    i32x4_t v = {0, 0, 0, 0};
    if (gr < rows_valid && gk < k_valid) {
      const bf16_t* p = KMAJOR ? base + (int64_t)gr * ld + gk : base + (int64_t)gk * ld + gr;
      v = *(const i32x4_t*)p;
    }
    reg[i] = v;
  }
}

template <int ROWS, bool KMAJOR>
__device__ __forceinline__ void store_slice(const i32x4_t* __restrict__ reg,
                                            bf16_t* __restrict__ tile, int tid) {
  using G = TileGeom<ROWS, KMAJOR>;
#pragma unroll
  for (int i = 0; i < G::PER_THREAD; ++i) {
    const int c = tid + 256 * i;
    int r, k;
    if (KMAJOR) { r = c / (BK / 8); k = (c % (BK / 8)) * 8; *(i32x4_t*)(tile + r * G::LD + k) = reg[i]; }
    else        { k = c / (ROWS / 8); r = (c % (ROWS / 8)) * 8; *(i32x4_t*)(tile + k * G::LD + r) = reg[i]; }
  }
}

// MFMA operand fragment: lane l gets row (r0 + l % 32), k = kk + 8 * (l / 32) .. + 7.
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ bf16x8_t read_frag(const bf16_t* __restrict__ tile, int r0, int kk, int lane) {
  using G = TileGeom<ROWS, KMAJOR>;
  if (KMAJOR) {
    return *(const bf16x8_t*)(tile + (r0 + (lane & 31)) * G::LD + kk + 8 * (lane >> 5));
  } else {
    // transpose read: the 16 lanes of a group pass the addresses of 4 k-rows x
    // 4 chunks of 4 rows; lane l of the group receives k-rows 0..3 of row l.
    const int gi = lane >> 4, r = lane & 15;
    const bf16_t* p = tile + (kk + 8 * (gi >> 1) + (r >> 2)) * G::LD + r0 + 16 * (gi & 1) + 4 * (r & 3);
    typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)p);
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * G::LD));
    union { struct { s16x4_t a, b; } s; bf16x8_t v; } u;
    u.s.a = lo; u.s.b = hi;
    return u.v;
  }
}

__device__ __forceinline__ int remap_xcd(int pid, int total) {
  const int base = total / NUM_XCD, rem = total % NUM_XCD;
  const int xcd = pid % NUM_XCD, idx = pid / NUM_XCD;
  return xcd * base + (xcd < rem ? xcd : rem) + idx;
}

template <int TM, int TN, bool XK, bool WK, bool F32OUT>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(GemmGroup grp, int total_tiles) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  using GX = TileGeom<BM, XK>;
  using GW = TileGeom<BN, WK>;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  constexpr int STAGE = GX::ELEMS + GW::ELEMS;   // stage s: X tile at s*STAGE, W tile after it

  // ---- which tile of which problem
  int pid = remap_xcd(blockIdx.x, total_tiles);
  int pi = 0, tiles_m = 0, tiles_n = 0;
  for (;; ++pi) {
    tiles_m = (grp.p[pi].M + BM - 1) / BM;
    tiles_n = (grp.p[pi].N + BN - 1) / BN;
    const int t = tiles_m * tiles_n;
    if (pid < t || pi + 1 == grp.count) break;
    pid -= t;
  }
  const GemmArgs& g = grp.p[pi];
  const int per_group = GROUP_M * tiles_n;
  const int first_m = (pid / per_group) * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int tm = first_m + (pid % per_group) % gsz;
  const int tn = (pid % per_group) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * (32 * TM), wn = (wave & 1) * (32 * TN);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  i32x4_t xr[GX::PER_THREAD], wr[GW::PER_THREAD];

#pragma unroll 1
  for (int seg = 0; seg < 2; ++seg) {
    const bf16_t* X = (const bf16_t*)(seg ? g.A2 : g.A);
    const bf16_t* W = (const bf16_t*)(seg ? g.B2 : g.B);
    const int K = seg ? g.K2 : g.K;
    const int64_t ldx = seg ? g.lda2 : g.lda, ldw = seg ? g.ldb2 : g.ldb;
    if (X == nullptr || K <= 0) continue;
    const int nk = (K + BK - 1) / BK;

    load_slice<BM, XK>(xr, X, ldx, m0, 0, g.M, K, tid);
    load_slice<BN, WK>(wr, W, ldw, n0, 0, g.N, K, tid);
    __syncthreads();                       // previous segment's readers are done
    store_slice<BM, XK>(xr, smem, tid);
    store_slice<BN, WK>(wr, smem + GX::ELEMS, tid);
    __syncthreads();

#pragma unroll 1
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1;
      const bool more = kt + 1 < nk;
      if (more) {
        load_slice<BM, XK>(xr, X, ldx, m0, (kt + 1) * BK, g.M, K, tid);
        load_slice<BN, WK>(wr, W, ldw, n0, (kt + 1) * BK, g.N, K, tid);
      }
      const bf16_t* xt = smem + cur * STAGE;
      const bf16_t* wt = xt + GX::ELEMS;
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        bf16x8_t xf[TM], wf[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) xf[i] = read_frag<BM, XK>(xt, wm + 32 * i, kk, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[j] = read_frag<BN, WK>(wt, wn + 32 * j, kk, lane);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], xf[i], acc[i][j], 0, 0, 0);
      }
      if (more) {
        store_slice<BM, XK>(xr, smem + (cur ^ 1) * STAGE, tid);
        store_slice<BN, WK>(wr, smem + (cur ^ 1) * STAGE + GX::ELEMS, tid);
      }
      __syncthreads();
    }
  }

  // ---- epilogue: lane holds C row m = .. + lane % 32; register e of tile (i, j)
  // holds column n = .. + 8 * (e / 4) + 4 * (lane / 32) + e % 4.
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm + 32 * i + (lane & 31);
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn + 32 * j + 8 * q + 4 * (lane >> 5);
        if (n >= g.N) continue;
        const float a0 = acc[i][j][4 * q], a1 = acc[i][j][4 * q + 1], a2 = acc[i][j][4 * q + 2],
                    a3 = acc[i][j][4 * q + 3];
        if (F32OUT) {
          float4 v = {a0, a1, a2, a3};
          *(float4*)((float*)g.C + (int64_t)m * g.ldc + n) = v;
        } else {
          uint2 v = {pack_bf16x2(a0, a1), pack_bf16x2(a2, a3)};
          *(uint2*)((bf16_t*)g.C + (int64_t)m * g.ldc + n) = v;
        }
      }
    }
  }
}

template <int TM, int TN, bool XK, bool WK, bool F32OUT>
static void launch_variant(const GemmGroup& grp, int total, hipStream_t s) {
  auto kern = gemm_bf16_kernel<TM, TN, XK, WK, F32OUT>;
  constexpr size_t smem =
      2 * (size_t)(TileGeom<64 * TM, XK>::ELEMS + TileGeom<64 * TN, WK>::ELEMS) * sizeof(bf16_t);
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(total), dim3(256), smem, s, grp, total);
}

template <int TM, int TN>
static void launch_tiles(const GemmGroup& grp, hipStream_t s) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  int total = 0;
  for (int i = 0; i < grp.count; ++i)
    total += ((grp.p[i].M + BM - 1) / BM) * ((grp.p[i].N + BN - 1) / BN);
  if (total == 0) return;
  const bool xk = grp.p[0].a_kmajor, wk = grp.p[0].b_kmajor, f32 = grp.p[0].c_is_f32;
  if (xk && !wk && !f32) launch_variant<TM, TN, true, false, false>(grp, total, s);
  else if (xk && wk && !f32) launch_variant<TM, TN, true, true, false>(grp, total, s);
  else if (!xk && !wk && !f32) launch_variant<TM, TN, false, false, false>(grp, total, s);
  else if (!xk && !wk && f32) launch_variant<TM, TN, false, false, true>(grp, total, s);
  else launch_gemm_bf16_scalar(grp, s, "gemm_bf16_scalar");   // no hot-path call lands here
}

// Every GEMM of a group must share storage orders and output type; the hot
// path only forms such groups.  Supported: X k-major with W either order
// (forward projections, input gradients), both row-major-in-k (weight grads).
void launch_gemm_bf16(const GemmGroup& grp, hipStream_t s, const char* name) {
  ProfScope ps(name, s);
  // tile choice: 256 x 256 when that still yields at least one tile per CU
  long tiles256 = 0;
  for (int i = 0; i < grp.count; ++i)
    tiles256 += (long)((grp.p[i].M + 255) / 256) * ((grp.p[i].N + 255) / 256);
  if (tiles256 >= 256) launch_tiles<4, 4>(grp, s);
  else launch_tiles<2, 2>(grp, s);
}

}  // namespace beagle
