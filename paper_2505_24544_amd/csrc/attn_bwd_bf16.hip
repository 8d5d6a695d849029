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
//      also computes delta and stores it, with -log2(e) * LSE, for kernel (2).
//
//  (2) dkv kernel  one workgroup = 128 keys of one (b, kv head), loop over the
//      H/G query heads of the group and over the query tiles that can see those
//      keys.  A lane owns ONE key: S = Q K^T and dP = dO V^T come out with
//      column j = lane % 32; P and dS go straight into the B operands of
//      dV^T += dO^T P and dK^T += Q^T dS.  LSE/delta of the tile's queries are
//      read from LDS (they index the accumulator registers here).
//
// Tiles go from HBM/L2 straight into one of two LDS stages while the other is
// consumed; the swizzled tile layout (attn_tiles.h) serves both the whole-row
// fragments (k = channel) and the transpose fragments (k = row) without bank
// conflicts.
//
// Mask: query p sees key j iff j < row_limit(p) iff p >= first_query_seeing(j).
// Key tiles beyond a workgroup's last limit / query tiles before a key tile's
// first viewer are never visited (whole-tile skipping).
#include "attn_tiles.h"

namespace beagle {
using namespace tiles;

namespace bwd {
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
constexpr int TILE = BJ * HD;            // one K or V tile
}  // namespace dqk

__global__ __launch_bounds__(256, 2) void attn_bwd_dq_bf16_kernel(AttnArgs a) {
  using namespace dqk;
  args_at_hand(a);
  __shared__ __attribute__((aligned(1024))) bf16_t stage0[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t stage1[2 * TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5, ql = lane & 31;
  const int nqt = (a.S + BQ - 1) / BQ;
  int row, tpos;
  map_block(blockIdx.x, a.H * a.B, row, tpos);
  const int qt = nqt - 1 - tpos;                  // heaviest (latest) query tiles first
  const int h = row % a.H, b = row / a.H, g = h / (a.H / a.G);
  const int q0 = qt * BQ, qw0 = q0 + wave * 32, q = qw0 + ql;
  const SeqView sv = seq_view(a, b);
  if (q0 >= sv.S) return;                         // packed batch: this entry is shorter than the longest one
  const bool q_ok = q < sv.S;
  const int qc = q_ok ? q : sv.S - 1;
  const int64_t qrow = ((sv.q0 + qc) * a.H + h) * HD;
  const bf16_t* Qg = (const bf16_t*)a.q + qrow;
  const bf16_t* Og = (const bf16_t*)a.o + qrow;
  const bf16_t* dOg = (const bf16_t*)a.dout + qrow;
  const int64_t kvs = (int64_t)a.G * HD;
  const __amdgpu_buffer_rsrc_t krs = rows_rsrc((const bf16_t*)a.k + (sv.kv0 * a.G + g) * HD, sv.L, kvs);
  const __amdgpu_buffer_rsrc_t vrs = rows_rsrc((const bf16_t*)a.v + (sv.kv0 * a.G + g) * HD, sv.L, kvs);
  const int64_t li = sv.lse0 + h * sv.lse_hs + qc;

  auto fetch = [&](bf16_t* st, int jt) {
    load_rows<BJ>(st, krs, kvs, jt * BJ, tid);
    load_rows<BJ>(st + TILE, vrs, kvs, jt * BJ, tid);
  };
  // The first K/V tile, the LSE and this lane's own rows are requested one behind the other and before the mask's
  // arithmetic: one trip to memory for all of them (measured per workgroup: 9 300 cycles until the rows are there,
  // 3 300 more when the LSE is only asked for then), with the integer divisions of the mask running meanwhile.  Tile 0
  // exists unless no query of the workgroup sees any key; then its rows are fetched for nothing.
  fetch(stage0, 0);
  const float lse = a.lse[li];
  bf16x8_t qf[8], dof[8], of[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    qf[s] = *(const bf16x8_t*)(Qg + 16 * s + 8 * hf);
    dof[s] = *(const bf16x8_t*)(dOg + 16 * s + 8 * hf);
    of[s] = *(const bf16x8_t*)(Og + 16 * s + 8 * hf);
  }
  __builtin_amdgcn_sched_barrier(0);

  const MaskParams mk = sample_mask(a, b);
  const int lim = q_ok ? row_limit(q, mk) : 0;
  const int wg_lim = row_limit(min(q0 + BQ, sv.S) - 1, mk);
  const int wave_hi = qw0 < sv.S ? row_limit(min(qw0 + 32, sv.S) - 1, mk) : 0;
  const int wave_lo = qw0 < sv.S ? row_limit(qw0, mk) : 0;
  const int ntiles = (wg_lim + BJ - 1) / BJ;
  __builtin_amdgcn_sched_barrier(0);

  float part = 0.f;
#pragma unroll
  for (int s = 0; s < 8; ++s) part += bwd::dot8(dof[s], of[s]);
  const float delta = half_pair_sum(part);
  if (q_ok && hf == 0) { a.delta[li] = delta; a.nlse2[li] = -LOG2E * lse; }   // blind rows: +inf, masked in the dK/dV kernel
  const float c2 = a.scale * LOG2E;
  const float lse2 = (lim > 0 ? lse : 0.f) * LOG2E;    // blind rows are fully masked below
  const FragOffs fo = make_frag_offs(lane);

  f32x16_t dq[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;

  auto tile_step = [&](const bf16_t* cur, bf16_t* nxt, int jt) {
    const int j0 = jt * BJ;
    if (j0 >= wave_hi) fetch(nxt, jt + 1);        // a wave that sees nothing of the tile only requests its share of the next
    if (j0 < wave_hi) {
      fetch(nxt, jt + 1);                         // issued between the MFMAs below
      const bf16_t* ks = cur;
      const bf16_t* vs = cur + TILE;
      f32x16_t st[2], dp[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) { st[jb][e] = 0.f; dp[jb][e] = 0.f; }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(ks, fo, jb, s), qf[s], st[jb], 0, 0, 0);
          dp[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(vs, fo, jb, s), dof[s], dp[jb], 0, 0, 0);
        }
      }
      pipeline_reads_mfma_loads<32, 1, 8>();
      __builtin_amdgcn_sched_barrier(0);
      // dS = P (dP - delta); key offsets inside the tile are compile-time constants, and only tiles that reach
      // past the smallest limit of the wave run the compares and selects (a scalar branch around them alone)
      float dsv[2][16];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(st[jb][e] * c2 - lse2);
          dsv[jb][e] = p * (dp[jb][e] - delta);
        }
      if (j0 + BJ > wave_lo) {
        const int rel = lim - j0 - 4 * hf;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (32 * jb + 8 * (e >> 2) + (e & 3) >= rel) dsv[jb][e] = 0.f;
      }
      uint32_t pk[2][8];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int e = 0; e < 16; e += 2) pk[jb][e >> 1] = cvt_pk(dsv[jb][e], dsv[jb][e + 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          union { uint32_t u[4]; bf16x8_t v; } sf;
#pragma unroll
          for (int i = 0; i < 4; ++i) sf.u[i] = pk[jb][4 * t + i];
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            dq[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(ks, fo, 32 * jb + 16 * t, cb), sf.v, dq[cb], 0, 0, 0);
        }
      pipeline_reads_mfma<16, 2>();
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmem();
    __syncthreads();
  };

  wait_vmem();
  __syncthreads();
  int jt = 0;
#pragma unroll 1
  for (; jt + 2 <= ntiles; jt += 2) {
    tile_step(stage0, stage1, jt);
    tile_step(stage1, stage0, jt + 1);
  }
  if (jt < ntiles) tile_step(stage0, stage1, jt);

  // ---- dQ rows out, through LDS (the stages are free: the last step, or the prologue, ended with a barrier)
  {
    uint2 pq[16];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd)
        pq[4 * cb + qd] = make_uint2(cvt_pk(dq[cb][4 * qd] * a.scale, dq[cb][4 * qd + 1] * a.scale),
                                     cvt_pk(dq[cb][4 * qd + 2] * a.scale, dq[cb][4 * qd + 3] * a.scale));
    store_rows_via_lds(stage0 + wave * 32 * HD, pq, lane, (bf16_t*)a.dq + ((sv.q0 + qw0) * a.H + h) * HD, (int64_t)a.H * HD,
                       sv.S - qw0);
  }
}

// ===========================================================================
// (2) dK and dV
// ===========================================================================
namespace dkv {
constexpr int BJ = 128, BQ = 64;
constexpr int TILE = BQ * HD;            // one Q or dO tile
}  // namespace dkv

__global__ __launch_bounds__(256, 1) void attn_bwd_dkv_bf16_kernel(AttnArgs a) {
  using namespace dkv;
  args_at_hand(a);
  __shared__ __attribute__((aligned(1024))) bf16_t stage0[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t stage1[2 * TILE];
  // [-log2(e) lse 64 | delta 64] of the stage's queries; waves 2 and 3 repeat the two requests into the second half,
  // which nobody reads, so that the request sequence has no branch and can be issued between MFMAs
  __shared__ __attribute__((aligned(256))) float stat0[4 * BQ];
  __shared__ __attribute__((aligned(256))) float stat1[4 * BQ];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5, jl = lane & 31;
  int row, jt;                                    // key tile 0 is seen by the most queries: heaviest first
  map_block(blockIdx.x, a.G * a.B, row, jt);
  const int g = row % a.G, b = row / a.G;
  const int rep = a.H / a.G;
  const int j0 = jt * BJ, jw0 = j0 + wave * 32, j = jw0 + jl;
  const SeqView sv = seq_view(a, b);
  if (j0 >= sv.L) return;                         // packed batch: this entry is shorter than the longest one
  const bool j_ok = j < sv.L;
  const int jc = j_ok ? j : sv.L - 1;
  const int64_t kvrow = ((sv.kv0 + jc) * a.G + g) * HD;
  const bf16_t* Kg = (const bf16_t*)a.k + kvrow;
  const bf16_t* Vg = (const bf16_t*)a.v + kvrow;
  const int64_t qs = (int64_t)a.H * HD;

  // This lane's K and V rows are requested before any of the mask's arithmetic, the first Q / dO tile as soon as the
  // first query tile is known, and the rest of that arithmetic (three more integer divisions) runs while they travel.
  bf16x8_t kf[8], vf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    kf[s] = *(const bf16x8_t*)(Kg + 16 * s + 8 * hf);
    vf[s] = *(const bf16x8_t*)(Vg + 16 * s + 8 * hf);
  }
  __builtin_amdgcn_sched_barrier(0);

  // first query that sees any key of the workgroup; below: this lane's key / any key of the wave / every key of the wave
  const MaskParams mk = sample_mask(a, b);
  const int wg_first = first_query_seeing(j0, mk);
  const int qt0 = wg_first / BQ;
  const int nqt = (sv.S + BQ - 1) / BQ;
  const int per_head = nqt > qt0 ? nqt - qt0 : 0;
  const int iters = per_head * rep;                 // (head, query tile) pairs, head-major
  int fq, wave_first, wave_all;                     // set behind the first tile's requests
  const float c2 = a.scale * LOG2E;
  const FragOffs fo = make_frag_offs(lane);

  f32x16_t dk[4], dv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[i][e] = 0.f; dv[i][e] = 0.f; }

  // Q / dO rows and the LSE / delta entries of tile `it`; rows and entries past
  // the sequence end arrive as zeros (zero Q and dO rows contribute nothing).
  int f_hh = 0, f_qt = qt0;                         // fetch cursor: head within the group, query tile
  int c_qt = qt0;                                   // compute cursor: query tile
  const int64_t head0 = sv.q0 * a.H + g * rep;
  const bf16_t* f_q = (const bf16_t*)a.q + head0 * HD;           // row 0 of the fetch cursor's head
  const bf16_t* f_do = (const bf16_t*)a.dout + head0 * HD;
  const float* f_stat = ((wave & 1) == 0 ? a.nlse2 : a.delta) + sv.lse0 + (g * rep) * sv.lse_hs;
  const int tile_bytes = sv.S > 0 ? (int)((((int64_t)sv.S - 1) * qs + HD) * 2) : 0;   // one head's Q (dO) rows of this entry
  auto fetch = [&](bf16_t* st, float* stat) {
    const int q0 = f_qt * BQ;
    const bool live = f_hh < rep;                    // past the last pair: empty descriptors, i.e. zeros
    const int tbytes = live ? tile_bytes : 0, sbytes = live ? sv.S * 4 : 0;
    load_rows<BQ>(st, __builtin_amdgcn_make_buffer_rsrc((void*)f_q, 0, tbytes, 0x00020000), qs, q0, tid);
    load_rows<BQ>(st + TILE, __builtin_amdgcn_make_buffer_rsrc((void*)f_do, 0, tbytes, 0x00020000), qs, q0, tid);
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc((void*)f_stat, 0, sbytes, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(srs, (lds_void_ptr)(stat + wave * BQ), 4, (q0 + lane) * 4, 0, 0, 0);
    // advance the cursor without branches
    const bool wrap = f_qt + 1 == nqt;
    const bool adv = wrap && f_hh + 1 < rep;
    f_qt = wrap ? qt0 : f_qt + 1;
    f_hh += wrap ? 1 : 0;
    f_q += adv ? HD : 0; f_do += adv ? HD : 0; f_stat += adv ? sv.lse_hs : 0;
  };

  auto tile_step = [&](const bf16_t* cur, const float* sl, bf16_t* nxt, float* nstat) {
    const int q0 = c_qt * BQ;
    if (++c_qt == nqt) c_qt = qt0;
    if (q0 + BQ <= wave_first) fetch(nxt, nstat);     // a wave that sees nothing of the tile only requests its share of the next
    if (q0 + BQ > wave_first) {                       // some query of the tile sees some key of the wave
      fetch(nxt, nstat);                              // issued between the first MFMAs below
      const bf16_t* qsm = cur;
      const bf16_t* dsm = cur + TILE;
      const int relq = fq - q0 - 4 * hf;    // query offsets inside the tile are compile-time constants
      // The two 32-query blocks of the tile go through  scores -> probabilities -> accumulation  one
      // phase apart, so that the exponentials and products of one block issue between the MFMAs of
      // the other (this kernel has one wave per SIMD: nothing else would fill the matrix pipe then).
      // Register e of block qb is query q0 + 32 qb + 8 (e/4) + 4 hf + e%4 ; column = this lane's key.
      {
        constexpr int VPM = 10;   // vector instructions of one block slotted in per MFMA of the other
        f32x16_t s2[2], dp[2];
        float4 l4[4], d4[4];
        uint32_t pp[2][8], pd[2][8];
        auto stats = [&](int qb) {
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const int r = 32 * qb + 8 * e4 + 4 * hf;
            l4[e4] = *(const float4*)(sl + r);
            d4[e4] = *(const float4*)(sl + BQ + r);
          }
        };
        auto scores = [&](int qb) {
#pragma unroll
          for (int e = 0; e < 16; ++e) { s2[qb][e] = 0.f; dp[qb][e] = 0.f; }
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            s2[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(qsm, fo, qb, s), kf[s], s2[qb], 0, 0, 0);
            dp[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(dsm, fo, qb, s), vf[s], dp[qb], 0, 0, 0);
          }
        };
        auto probs = [&](int qb) {
          float pv[16];
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const float ls[4] = {l4[e4].x, l4[e4].y, l4[e4].z, l4[e4].w};
#pragma unroll
            for (int u = 0; u < 4; ++u) pv[4 * e4 + u] = __builtin_amdgcn_exp2f(__builtin_fmaf(s2[qb][4 * e4 + u], c2, ls[u]));
          }
          // The per-element predicate only where some key of the wave is hidden from some query of the block (a
          // scalar branch around the compares and selects alone: the kernel is bound by instruction issue, and a
          // second copy of the whole body made the register allocator shuffle the accumulators).  A blind query
          // (-log2(e) LSE = +inf, p = +inf) is below fq for every key, so its block always comes through here.
          if (q0 + 32 * qb < wave_all) {
#pragma unroll
            for (int e = 0; e < 16; ++e)
              if (32 * qb + 8 * (e >> 2) + (e & 3) < relq) pv[e] = 0.f;
          }
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const float dl[4] = {d4[e4].x, d4[e4].y, d4[e4].z, d4[e4].w};
            float dsv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) dsv[u] = pv[4 * e4 + u] * (dp[qb][4 * e4 + u] - dl[u]);
            pp[qb][2 * e4] = cvt_pk(pv[4 * e4], pv[4 * e4 + 1]); pp[qb][2 * e4 + 1] = cvt_pk(pv[4 * e4 + 2], pv[4 * e4 + 3]);
            pd[qb][2 * e4] = cvt_pk(dsv[0], dsv[1]); pd[qb][2 * e4 + 1] = cvt_pk(dsv[2], dsv[3]);
          }
        };
        auto accum = [&](int qb) {
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            union { uint32_t u[4]; bf16x8_t v; } pf, sf;
#pragma unroll
            for (int i = 0; i < 4; ++i) { pf.u[i] = pp[qb][4 * t + i]; sf.u[i] = pd[qb][4 * t + i]; }
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
              dv[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(dsm, fo, 32 * qb + 16 * t, cb), pf.v, dv[cb], 0, 0, 0);
              dk[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(qsm, fo, 32 * qb + 16 * t, cb), sf.v, dk[cb], 0, 0, 0);
            }
          }
        };
        scores(0);
        pipeline_reads_mfma_loads<16, 1, 9>();
        __builtin_amdgcn_sched_barrier(0);
        stats(0);
        scores(1);
        probs(0);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
        pipeline_reads_mfma_valu<16, 1, VPM>();
        __builtin_amdgcn_sched_barrier(0);
        stats(1);
        accum(0);
        probs(1);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
        pipeline_reads_mfma_valu<16, 2, VPM>();
        __builtin_amdgcn_sched_barrier(0);
        accum(1);
        pipeline_reads_mfma<16, 2>();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    wait_vmem();
    __syncthreads();
  };

  if (iters > 0) fetch(stage0, stat0);
  __builtin_amdgcn_sched_barrier(0);
  fq = j_ok ? first_query_seeing(j, mk) : sv.S;
  wave_first = jw0 < sv.L ? first_query_seeing(jw0, mk) : sv.S;
  wave_all = jw0 < sv.L ? first_query_seeing(min(jw0 + 32, sv.L) - 1, mk) : sv.S;
  __builtin_amdgcn_sched_barrier(0);
  wait_vmem();
  __syncthreads();
  int it = 0;
#pragma unroll 1
  for (; it + 2 <= iters; it += 2) {
    tile_step(stage0, stat0, stage1, stat1);
    tile_step(stage1, stat1, stage0, stat0);
  }
  if (it < iters) tile_step(stage0, stat0, stage1, stat1);

  // ---- dK, dV rows out, through LDS (both stages are free: the last step ended with the requests landed and a barrier)
  {
    uint2 pk[16], pv[16];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        pk[4 * cb + qd] = make_uint2(cvt_pk(dk[cb][4 * qd] * a.scale, dk[cb][4 * qd + 1] * a.scale),
                                     cvt_pk(dk[cb][4 * qd + 2] * a.scale, dk[cb][4 * qd + 3] * a.scale));
        pv[4 * cb + qd] = make_uint2(cvt_pk(dv[cb][4 * qd], dv[cb][4 * qd + 1]), cvt_pk(dv[cb][4 * qd + 2], dv[cb][4 * qd + 3]));
      }
    const int64_t wrow = ((sv.kv0 + jw0) * a.G + g) * HD;               // row of the wave's first key
    const int64_t kvs = (int64_t)a.G * HD;
    store_rows_via_lds(stage0 + wave * 32 * HD, pk, lane, (bf16_t*)a.dk + wrow, kvs, sv.L - jw0);
    store_rows_via_lds(stage1 + wave * 32 * HD, pv, lane, (bf16_t*)a.dv + wrow, kvs, sv.L - jw0);
  }
}

// workspace: the pre-scaled LSE array, as large as delta
size_t attn_bwd_bf16_ws_bytes(const AttnArgs& a) { return (size_t)a.B * a.H * a.S * sizeof(float); }

void launch_attn_bwd_bf16(const AttnArgs& args, void* ws, hipStream_t s) {
  AttnArgs a = args;
  a.nlse2 = (float*)ws;
  {
    ProfScope ps("attn_bwd_dq_bf16", s);
    dim3 grid(((a.S + dqk::BQ - 1) / dqk::BQ) * a.H * a.B);
    hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel, grid, dim3(256), 0, s, a);
  }
  {
    ProfScope ps("attn_bwd_dkv_bf16", s);
    dim3 grid(((a.L + dkv::BJ - 1) / dkv::BJ) * a.G * a.B);
    hipLaunchKernelGGL(attn_bwd_dkv_bf16_kernel, grid, dim3(256), 0, s, a);
  }
}

}  // namespace beagle
