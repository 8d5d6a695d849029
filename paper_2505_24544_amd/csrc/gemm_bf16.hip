// bf16 GEMM on the gfx950 matrix cores: C[M,N] = X * W (+ X2 * W2), float
// accumulation, for the Q/K/V/output projections of Eq. 2 and every
// projection-shaped contraction of the backward pass.
//
// Design
//   * One workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile of C; each
//     wave owns (32*TM) x (32*TN) of it as TM x TN accumulators of the
//     v_mfma_f32_32x32x16_bf16 instruction.
//   * The k loop walks BK = 64 at a time through two LDS stages.  Slices go
//     from HBM/L2 straight into LDS (buffer_load ... lds, 16 bytes per lane):
//     no staging registers, no ds_write, and out-of-range chunks arrive as
//     zeros through the buffer descriptor's range check.  The loads of slice
//     t+1 are issued before the MFMAs of slice t; one vmcnt wait + barrier per
//     slice.  The two stages are two separate __shared__ arrays so that the
//     compiler can tell a fragment read of one stage from an in-flight load
//     into the other.
//   * Each operand tile sits in LDS in the order it has in HBM (a lane's 16
//     bytes land at wave_base + 16 * lane), with an XOR swizzle chosen on the
//     GLOBAL side (which chunk a lane fetches) so that reads are conflict free:
//       k-contiguous operand  -> rows of 128 B; chunk c of row r is stored at
//                                chunk c ^ ((r >> 1) & 7); a fragment is one
//                                ds_read_b128;
//       row-contiguous operand-> k-rows of ROWS*2 B; chunk c of k-row k is
//                                stored at chunk c ^ ((k & 3) << 2); a fragment
//                                is two ds_read_b64_tr_b16 (the LDS transpose
//                                read), which hand every lane four consecutive
//                                k of its own row.
//   * Fragments are double-buffered in registers: those of k step s+1 are read
//     from LDS before the MFMAs of step s are issued.
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
#include <stdio.h>
#include <stdlib.h>
#include "common.h"

namespace beagle {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr int BK = 64;
constexpr int GROUP_M = 4;
constexpr int NUM_XCD = 8;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, int64_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, (int)bytes, 0x00020000);
}

// One BK slice of one operand, HBM -> LDS.  Chunk q = tid + 256 i of the tile
// (16 bytes) lands at tile + 16 q; which global chunk it is follows from the
// swizzle.
//   KMAJOR : element (row r, k) at base[r * ld + k]   (buffer = rows * ld elements)
//   !KMAJOR: element (row r, k) at base[k * ld + r]   (buffer = K * ld elements)
// k beyond K must read as zero: for !KMAJOR that is past the end of the buffer;
// for KMAJOR the launcher requires K % BK == 0.  Rows beyond the matrix only
// feed output rows/columns that are never stored, so whatever they read (zero
// past the end, or a neighbouring row) is harmless.
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ void load_slice(bf16_t* tile, __amdgpu_buffer_rsrc_t rsrc, int64_t ld, int row0, int k0,
                                           int tid) {
  constexpr int PER_THREAD = ROWS * BK / 8 / 256;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) {
    const int q = tid + 256 * i;
    int off;
    if (KMAJOR) {
      const int r = q >> 3, c = (q & 7) ^ ((r >> 1) & 7);
      off = (int)(((int64_t)(row0 + r) * ld + k0 + 8 * c) * 2);
    } else {
      constexpr int CPR = ROWS / 8;
      const int k = q / CPR, c = (q % CPR) ^ ((k & 3) << 2);
      off = (int)(((int64_t)(k0 + k) * ld + row0 + 8 * c) * 2);
    }
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(tile + (i * 4 + wave) * 512), 16, off, 0, 0, 0);
  }
}

// Per-lane element offsets of an operand's fragments inside its tile, computed
// once per kernel.  Everything that varies inside the k loop (the 32-row block
// for k-contiguous tiles, the k step for both) is then a compile-time constant
// added to one of these, i.e. an immediate offset of the LDS read.
//   KMAJOR : o[ks]  = row (l % 32), swizzled chunk of k step ks       (+ 32-row block * BK)
//   !KMAJOR: o[blk] = k-row (8 (l/32) + (l%16)/4), swizzled column of block blk   (+ k step * 16 * ROWS)
template <int ROWS, bool KMAJOR, int NBLK>
struct FragOffs {
  int o[KMAJOR ? BK / 16 : NBLK];
  __device__ __forceinline__ void init(int lane, int r0) {
    if (KMAJOR) {
      const int ql = lane & 31, hf = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) o[ks] = (r0 + ql) * BK + (((2 * ks + hf) ^ ((ql >> 1) & 7)) << 3);
    } else {
      const int gi = lane >> 4, r16 = lane & 15;
      const int kr = 8 * (gi >> 1) + (r16 >> 2);
#pragma unroll
      for (int b = 0; b < NBLK; ++b) {
        const int col = r0 + 32 * b + 16 * (gi & 1) + 4 * (r16 & 3);
        o[b] = kr * ROWS + ((((col >> 3) ^ ((kr & 3) << 2)) << 3) | (col & 7));
      }
    }
  }
};

// MFMA operand fragment: lane l gets row (r0 + 32 blk + l % 32), k = 16 ks + 8 * (l / 32) .. + 7.
template <int ROWS, bool KMAJOR, int NBLK>
__device__ __forceinline__ bf16x8_t read_frag(const bf16_t* tile, const FragOffs<ROWS, KMAJOR, NBLK>& f, int blk, int ks) {
  if (KMAJOR) {
    return *(const bf16x8_t*)(tile + blk * 32 * BK + f.o[ks]);
  } else {
    // transpose read: the 16 lanes of a group pass the addresses of 4 k-rows x
    // 4 pieces of 4 rows; lane l of the group receives k-rows 0..3 of row l.
    const bf16_t* p = tile + ks * 16 * ROWS + f.o[blk];
    union { struct { s16x4_t a, b; } s; bf16x8_t v; } u;
    u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
    u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * ROWS));
    return u.v;
  }
}

// Workgroup id -> (problem, tile index inside the problem).  Ids are dealt
// round-robin to the 8 XCDs; every problem's tiles are split evenly over the
// XCDs (contiguous runs, so neighbouring tiles share an L2), and an XCD walks
// the problems in order.  Remainder tiles of successive problems go to
// successive XCDs, which keeps the per-XCD totals equal to what the hardware
// deals out.  Problems of different depth (dXkv has twice the k of dXq) are thus
// balanced across XCDs instead of being concentrated on some of them.
__device__ __forceinline__ void map_tile(int pid, const int* tiles, int count, int& prob, int& local) {
  const int c = pid % NUM_XCD;
  int idx = pid / NUM_XCD, off = 0;
  prob = count - 1; local = 0;
  for (int p = 0; p < count; ++p) {
    const int base = tiles[p] / NUM_XCD, rem = tiles[p] % NUM_XCD;
    const int r = (c - off + NUM_XCD) % NUM_XCD;
    const int cnt = base + (r < rem ? 1 : 0);
    if (idx < cnt || p + 1 == count) { prob = p; local = r * base + (r < rem ? r : rem) + idx; return; }
    idx -= cnt;
    off = (off + rem) % NUM_XCD;
  }
}

// RES: some problem of the group has a residual operand R (a separate instantiation, so that the kernels
// without one keep their register allocation).
template <int TM, int TN, bool XK, bool WK, bool F32OUT, bool RES>
__global__ __launch_bounds__(256, TM * TN >= 16 ? 1 : 2) void gemm_bf16_kernel(GemmGroup grp, int total_tiles) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int XE = BM * BK, WE = BN * BK;      // elements per operand tile
  __shared__ __attribute__((aligned(1024))) bf16_t stage0[XE + WE];
  __shared__ __attribute__((aligned(1024))) bf16_t stage1[XE + WE];

  // ---- which tile of which problem
  int ntile[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    ntile[i] = i < grp.count ? ((grp.p[i].M + BM - 1) / BM) * ((grp.p[i].N + BN - 1) / BN) : 0;
  int pi, pid;
  map_tile(blockIdx.x, ntile, grp.count, pi, pid);
  const GemmArgs& g = grp.p[pi];
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  (void)total_tiles;
  const int per_group = GROUP_M * tiles_n;
  const int first_m = (pid / per_group) * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int tm = first_m + (pid % per_group) % gsz;
  const int tn = (pid % per_group) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave >> 1) * (32 * TM), wn = (wave & 1) * (32 * TN);

  FragOffs<BM, XK, TM> xo;
  FragOffs<BN, WK, TN> wo;
  xo.init(lane, wm);
  wo.init(lane, wn);

  // The accumulators are cleared behind the first segment's first requests, not ahead of them: 256 register
  // writes per lane are 2 000 cycles that the first round trip to memory can hide.
  f32x16_t acc[TM][TN];
  auto clear_acc = [&]() {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  };
  bool fresh = true;

#pragma unroll 1
  for (int seg = 0; seg < 2; ++seg) {
    const bf16_t* X = (const bf16_t*)(seg ? g.A2 : g.A);
    const bf16_t* W = (const bf16_t*)(seg ? g.B2 : g.B);
    const int K = seg ? g.K2 : g.K;
    const int64_t ldx = seg ? g.lda2 : g.lda, ldw = seg ? g.ldb2 : g.ldb;
    if (X == nullptr || K <= 0) continue;
    const int nk = (K + BK - 1) / BK;
    const __amdgpu_buffer_rsrc_t xrs = make_rsrc(X, (int64_t)(XK ? g.M : K) * ldx * 2);
    const __amdgpu_buffer_rsrc_t wrs = make_rsrc(W, (int64_t)(WK ? g.N : K) * ldw * 2);

    bf16x8_t xf[2][TM], wf[2][TN];
    auto fetch_x = [&](bf16_t* st, int k0) { load_slice<BM, XK>(st, xrs, ldx, m0, k0, tid); };
    auto fetch_w = [&](bf16_t* st, int k0) { load_slice<BN, WK>(st + XE, wrs, ldw, n0, k0, tid); };
    auto frags = [&](const bf16_t* st, int fb, int ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) xf[fb][i] = read_frag<BM, XK, TM>(st, xo, i, ks);
#pragma unroll
      for (int j = 0; j < TN; ++j) wf[fb][j] = read_frag<BN, WK, TN>(st + XE, wo, j, ks);
    };
    auto mfmas = [&](int fb) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[fb][j], xf[fb][i], acc[i][j], 0, 0, 0);
    };
    constexpr int NSTEP = BK / 16;                                      // k steps per slice (4)
    constexpr int NREADS = (XK ? TM : 2 * TM) + (WK ? TN : 2 * TN);     // LDS reads per k step
    constexpr int XLOADS = BM * BK / 8 / 256, WLOADS = BN * BK / 8 / 256;   // HBM->LDS loads per thread per slice
    static_assert(NSTEP == 4 && NREADS % 2 == 0 && NREADS / 2 <= TM * TN, "issue pattern below assumes this");
    static_assert(XLOADS <= TM * TN && WLOADS <= TM * TN, "one load per MFMA at most");
    // One k slice.  On entry: slice kt is visible in `cur` and its step-0 fragments are in
    // registers; the X half of slice kt+1 is already on its way into `nxt`.
    //   step 0    : MFMAs + LDS reads of step 1 + the W half of slice kt+1 (one load per MFMA)
    //   steps 1,2 : MFMAs + LDS reads of the next step
    //   wait for this thread's loads, barrier: slice kt+1 visible, nobody reads `cur` any more
    //   step 3    : MFMAs from registers + first fragment reads of slice kt+1 + the X half of
    //               slice kt+2 into `cur`
    // so every HBM->LDS load is issued at least two k steps (>= 1000 cycles) before it is
    // waited for, and the in-order wave never waits on a queue while the MFMA pipe is idle.
    auto slice = [&](bf16_t* cur, bf16_t* nxt, int kt) {
      fetch_w(nxt, (kt + 1) * BK);    // past the last slice these fetch zeros / unused rows: harmless
#pragma unroll
      for (int ks = 0; ks < NSTEP - 1; ++ks) {
        const int fb = ks & 1;
        frags(cur, fb ^ 1, ks + 1);
        mfmas(fb);
#pragma unroll
        for (int t = 0; t < TM * TN; ++t) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (t < NREADS / 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          if (ks == 0 && t < WLOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this thread's chunks of the next slice are in LDS
      __syncthreads();                      // everyone's are, and everyone is done reading `cur`
      frags(nxt, 0, 0);
      fetch_x(cur, (kt + 2) * BK);
      mfmas((NSTEP - 1) & 1);
#pragma unroll
      for (int t = 0; t < TM * TN; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (t < NREADS / 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        if (t < XLOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      }
    };

    __syncthreads();                        // previous segment: all reads done, both stages free
    fetch_x(stage0, 0);
    fetch_w(stage0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (fresh) { clear_acc(); fresh = false; }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    frags(stage0, 0, 0);
    fetch_x(stage1, BK);
    int kt = 0;
#pragma unroll 1
    for (; kt + 2 <= nk; kt += 2) {
      slice(stage0, stage1, kt);
      slice(stage1, stage0, kt + 1);
    }
    if (kt < nk) slice(stage0, stage1, kt);
    __builtin_amdgcn_s_waitcnt(0x0F70);     // drain the look-ahead loads before the stages are reused
  }
  if (fresh) clear_acc();                   // no segment at all: C = 0 (+ residual)

  // ---- residual operand: its tile goes HBM -> LDS in one burst (both stages are free now), so that the
  // epilogue below does not pay one HBM round trip per store.  Chunk q = tid + 256 i (16 bytes) of the tile
  // lands at 16 q; chunk position pc of row r holds global chunk pc ^ (r % CPR), which spreads the epilogue's
  // same-column reads of 32 different rows over the banks.  The upper half of the rows lives in stage1.
  constexpr int CPR = BN / 8;                      // 16-byte chunks per tile row
  constexpr int RLOADS = BM * CPR / 256;           // per thread
  const bool with_res = RES && !F32OUT && g.R != nullptr;
  if (with_res) {
    static_assert((BM / 2) * BN <= XE + WE, "half of the residual tile must fit one stage");
    __syncthreads();                               // every wave is done reading the operand stages
    const __amdgpu_buffer_rsrc_t rrs = make_rsrc(g.R, (int64_t)g.M * g.ldr * 2);
#pragma unroll
    for (int i = 0; i < RLOADS; ++i) {
      const int q = tid + 256 * i, r = q / CPR, c = (q % CPR) ^ (r & (CPR - 1));
      const int off = (int)(((int64_t)(m0 + r) * g.ldr + n0 + 8 * c) * 2);
      bf16_t* st = i < RLOADS / 2 ? stage0 : stage1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rrs, (lds_void_ptr)(st + ((i % (RLOADS / 2)) * 4 + wave) * 512), 16, off,
                                               0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }

  // ---- epilogue: lane holds C row m = .. + lane % 32; register e of tile (i, j)
  // holds column n = .. + 8 * (e / 4) + 4 * (lane / 32) + e % 4.
  if constexpr (F32OUT) {
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
          float4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *(float4*)((float*)g.C + (int64_t)m * g.ldc + n) = v;
        }
      }
    }
  } else {
    // bf16 output.  Straight from the registers a store instruction would carry 16 bytes for each of 32 rows, and
    // the workgroup -- the only one on its CU -- spent 15 % of its life issuing them (measured: 27 500 cycles per
    // 256 x 256 tile against 2 350 per k slice).  Each wave therefore transposes its part of the tile through a
    // patch of LDS of its own (the operand stages are free now; two patches per stage) and writes whole row
    // segments: 16 bytes per lane, 64 / CPW rows per instruction.  Patch rows hold CPW 16-byte chunks; chunk c
    // of row r sits at position c ^ (r % CPW), which spreads the column-wise writes over the banks.
    constexpr int CPW = 4 * TN;                      // chunks per patch row (32 TN columns)
    constexpr int PROWS = 32 * TM;                   // patch rows
    constexpr int RPI = 64 / CPW;                    // rows per store instruction
    static_assert(CPW <= 64 && 64 % CPW == 0 && PROWS % RPI == 0, "patch rows must tile a wave");
    static_assert(2 * PROWS * CPW * 8 <= XE + WE, "two patches per stage");
    if (with_res) {
      // the residual tile occupies the stages: take it into the accumulators first, then let go of it
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int rt = wm + 32 * i + (lane & 31);      // row inside the tile
        const bf16_t* rrow = (rt < BM / 2 ? stage0 : stage1) + (rt % (BM / 2)) * BN;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int ct = wn + 32 * j + 8 * q;        // first column of this 8-column chunk inside the tile
            const uint2 r = *(const uint2*)(rrow + (((ct >> 3) ^ (rt & (CPR - 1))) << 3) + 4 * (lane >> 5));
            acc[i][j][4 * q] += __uint_as_float(r.x << 16); acc[i][j][4 * q + 1] += __uint_as_float(r.x & 0xffff0000u);
            acc[i][j][4 * q + 2] += __uint_as_float(r.y << 16); acc[i][j][4 * q + 3] += __uint_as_float(r.y & 0xffff0000u);
          }
      }
    }
    __syncthreads();                                 // every wave is done reading the stages
    bf16_t* patch = (wave < 2 ? stage0 : stage1) + (wave & 1) * (PROWS * CPW * 8);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int pr = 32 * i + (lane & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 v = {pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]), pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3])};
          *(uint2*)(patch + pr * (CPW * 8) + (((4 * j + q) ^ (pr & (CPW - 1))) << 3) + 4 * (lane >> 5)) = v;
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own writes have landed; no other wave touches its patch
    const int pp = lane % CPW, rsub = lane / CPW;
#pragma unroll
    for (int it = 0; it < PROWS / RPI; ++it) {
      const int pr = it * RPI + rsub;
      const uint4 v = *(const uint4*)(patch + pr * (CPW * 8) + pp * 8);
      const int m = m0 + wm + pr, n = n0 + wn + 8 * (pp ^ (pr & (CPW - 1)));
      if (m < g.M && n < g.N) { typedef unsigned int nt_u32x4 __attribute__((ext_vector_type(4))); const nt_u32x4 w = {v.x, v.y, v.z, v.w}; __builtin_nontemporal_store(w, (nt_u32x4*)((bf16_t*)g.C + (int64_t)m * g.ldc + n)); }
    }
  }
}

template <int TM, int TN, bool XK, bool WK, bool F32OUT, bool RES = false>
static void launch_variant(const GemmGroup& grp, int total, hipStream_t s) {
  hipLaunchKernelGGL((gemm_bf16_kernel<TM, TN, XK, WK, F32OUT, RES>), dim3(total), dim3(256), 0, s, grp, total);
}

// What the MFMA kernel needs of a group (checked by the entry points before anything is enqueued, see
// gemm_bf16_supported): k-contiguous operands with K a multiple of the k slice, every operand (and the residual)
// addressable through a 32-bit buffer descriptor, and one of the storage-order combinations instantiated below.
static bool group_fits(const GemmGroup& grp) {
  if (grp.count < 1 || grp.count > 4) return false;
  const bool xk = grp.p[0].a_kmajor, wk = grp.p[0].b_kmajor, f32 = grp.p[0].c_is_f32;
  const int64_t lim = (int64_t)1 << 31;
  bool res = false;
  for (int i = 0; i < grp.count; ++i) {
    const GemmArgs& q = grp.p[i];
    if ((bool)q.a_kmajor != xk || (bool)q.b_kmajor != wk || (bool)q.c_is_f32 != f32) return false;
    if (q.R) { res = true; if ((int64_t)q.M * q.ldr * 2 >= lim) return false; }
    if ((xk || wk) && (q.K % BK || (q.A2 && q.K2 % BK))) return false;
    if ((int64_t)(xk ? q.M : q.K) * q.lda * 2 >= lim || (int64_t)(wk ? q.N : q.K) * q.ldb * 2 >= lim) return false;
    if (q.A2 && ((int64_t)(xk ? q.M : q.K2) * q.lda2 * 2 >= lim || (int64_t)(wk ? q.N : q.K2) * q.ldb2 * 2 >= lim)) return false;
  }
  if (res) return xk && !f32;
  return (xk && !f32) || (!xk && !wk);
}
bool gemm_bf16_supported(const GemmGroup& grp) { return group_fits(grp); }

template <int TM, int TN>
static void launch_tiles(const GemmGroup& grp, hipStream_t s) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  int total = 0;
  for (int i = 0; i < grp.count; ++i)
    total += ((grp.p[i].M + BM - 1) / BM) * ((grp.p[i].N + BN - 1) / BN);
  if (total == 0) return;
  const bool xk = grp.p[0].a_kmajor, wk = grp.p[0].b_kmajor, f32 = grp.p[0].c_is_f32;
  bool res = false;
  for (int i = 0; i < grp.count; ++i) if (grp.p[i].R) res = true;
  if (!group_fits(grp)) {
    // The entry points refuse such problems with BEAGLE_ERR_UNSUPPORTED before they enqueue anything; there is no
    // slower kernel to fall back to.  Getting here is a bug in the library's own host code.
    fprintf(stderr, "beagle_xattn: internal error: GEMM group outside the MFMA kernel's domain reached the launcher\n");
    abort();
  }
  if (res && !wk) launch_variant<TM, TN, true, false, false, true>(grp, total, s);
  else if (res) launch_variant<TM, TN, true, true, false, true>(grp, total, s);
  else if (xk && !wk) launch_variant<TM, TN, true, false, false>(grp, total, s);
  else if (xk) launch_variant<TM, TN, true, true, false>(grp, total, s);
  else if (!f32) launch_variant<TM, TN, false, false, false>(grp, total, s);
  else launch_variant<TM, TN, false, false, true>(grp, total, s);
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

template <bool F32OUT>
__global__ __launch_bounds__(256) void sum_pairs_kernel(SumPairArgs p, int64_t n4) {
  const int t = blockIdx.y;
  const float4* a = (const float4*)p.a[t];
  const float4* b = (const float4*)p.b[t];
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    const float4 x = a[i], y = b[i];
    const float4 v = {x.x + y.x, x.y + y.y, x.z + y.z, x.w + y.w};
    if (F32OUT) ((float4*)p.out[t])[i] = v;
    else ((uint2*)p.out[t])[i] = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
  }
}
void launch_sum_pairs(const SumPairArgs& p, int64_t n, bool out_f32, hipStream_t s, const char* name) {
  ProfScope ps(name, s);
  const int64_t n4 = n / 4;
  const dim3 grid((unsigned)((n4 + 255) / 256 < 2048 ? (n4 + 255) / 256 : 2048), p.count);
  if (out_f32) hipLaunchKernelGGL(sum_pairs_kernel<true>, grid, dim3(256), 0, s, p, n4);
  else hipLaunchKernelGGL(sum_pairs_kernel<false>, grid, dim3(256), 0, s, p, n4);
}

}  // namespace beagle
