// Flash-style forward of the block-masked cross-attention (Eq. 2 with the
// window mask of section 4.2) for bf16, head width 128, on gfx950 MFMA.
//
// One workgroup (4 waves) owns 128 queries of one (batch, head); each wave owns
// 32 of them.  Key/value tiles of 64 rows go from HBM/L2 straight into one of
// two LDS stages (see attn_tiles.h) while the other stage is consumed.
//
// Everything is computed transposed so that a lane owns ONE query:
//   S^T[j][q] = sum_c K[j][c] Q[q][c]     A operand = K rows   (ds_read_b128)
//                                          B operand = Q rows   (registers)
//   O^T[c][q] = sum_j V[j][c] P^T[j][q]   A operand = V^T      (ds_read_b64_tr_b16)
//                                          B operand = P^T, taken straight from
//                                          the S^T accumulator registers
// With the 32x32 MFMA output layout a lane holds column q = lane % 32, so the
// row max / row sum of the online softmax are reductions over the lane's own
// registers plus one exchange with lane ^ 32, and rescaling O is a per-lane
// scalar multiply.  The accumulator-to-operand hand-over of P needs no LDS
// round trip: the k index of the second MFMA is an arbitrary labelling of the
// 16 keys of a step, so V^T is simply fetched in the order the S^T registers
// already have.
//
// Mask: query p sees keys j < row_limit(p).  The loop over key tiles stops at
// the last tile any query of the workgroup can see (whole-tile skipping); only
// tiles that straddle a wave's limits evaluate the per-element predicate.
#include <type_traits>
#include "attn_tiles.h"

namespace beagle {
using namespace tiles;

namespace fwd {
constexpr int BQ = 128;           // queries per workgroup
constexpr int BJ = 64;            // keys per tile
constexpr int TILE = BJ * HD;     // elements of one K or V tile
constexpr float RESCALE_LOG2 = 8.f;
}  // namespace fwd

__global__ __launch_bounds__(256, 2) void attn_fwd_bf16_kernel(AttnArgs a) {
  using namespace fwd;
  args_at_hand(a);
  __shared__ __attribute__((aligned(1024))) bf16_t stage0[2 * TILE];
  __shared__ __attribute__((aligned(1024))) bf16_t stage1[2 * TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5, ql = lane & 31;
  const int nqt = (a.S + BQ - 1) / BQ;
  int row, tpos;
  map_block(blockIdx.x, a.H * a.B, row, tpos);
  const int qt = nqt - 1 - tpos;                  // heaviest (latest) query tiles first
  const int h = row % a.H, b = row / a.H;
  const int g = h / (a.H / a.G);
  const int q0 = qt * BQ;
  const SeqView sv = seq_view(a, b);
  if (q0 >= sv.S) return;                         // packed batch: this entry is shorter than the longest one
  const int qw0 = q0 + wave * 32;                 // first query of this wave
  const int q = qw0 + ql;                         // this lane's query
  const bool q_ok = q < sv.S;
  const int qc = q_ok ? q : sv.S - 1;

  const bf16_t* Qg = (const bf16_t*)a.q + ((sv.q0 + qc) * a.H + h) * HD;
  const int64_t kvs = (int64_t)a.G * HD;
  const __amdgpu_buffer_rsrc_t krs = rows_rsrc((const bf16_t*)a.k + (sv.kv0 * a.G + g) * HD, sv.L, kvs);
  const __amdgpu_buffer_rsrc_t vrs = rows_rsrc((const bf16_t*)a.v + (sv.kv0 * a.G + g) * HD, sv.L, kvs);

  // The first K/V tile and this lane's Q row are requested before the mask's arithmetic (several integer divisions):
  // the trip to memory and the arithmetic run side by side.  Tile 0 exists unless no query of the workgroup sees any
  // key; then its rows are fetched for nothing (they are inside the tensors either way).
  auto fetch = [&](bf16_t* st, int jt) {
    load_rows<BJ>(st, krs, kvs, jt * BJ, tid);
    load_rows<BJ>(st + TILE, vrs, kvs, jt * BJ, tid);
  };
  fetch(stage0, 0);
  // Q fragments: B operand, lane holds Q[q][16*s + 8*hf .. +7]
  bf16x8_t qf[HD / 16];
#pragma unroll
  for (int s = 0; s < HD / 16; ++s) qf[s] = *(const bf16x8_t*)(Qg + 16 * s + 8 * hf);
  __builtin_amdgcn_sched_barrier(0);

  const MaskParams mk = sample_mask(a, b);
  const int lim = q_ok ? row_limit(q, mk) : 0;                     // keys visible to this lane's query
  const int q_last = min(q0 + BQ, sv.S) - 1;
  const int wg_lim = row_limit(q_last, mk);                    // limits never decrease with p
  const int w_last = min(qw0 + 32, sv.S) - 1;
  const int wave_hi = qw0 < sv.S ? row_limit(w_last, mk) : 0;   // largest limit in this wave
  const int wave_lo = qw0 < sv.S ? row_limit(qw0, mk) : 0;      // smallest
  const int ntiles = (wg_lim + BJ - 1) / BJ;

  f32x16_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float c2 = a.scale * LOG2E;               // scores are kept raw; exp2((s - m) * c2)
  const FragOffs fo = make_frag_offs(lane);

  auto tile_step = [&](const bf16_t* cur, bf16_t* nxt, int jt) {
    const int j0 = jt * BJ;
    if (j0 >= wave_hi) fetch(nxt, jt + 1);        // a wave that sees nothing of the tile only requests its share of the next
    if (j0 < wave_hi) {                           // wave-uniform: this wave sees part of the tile
      fetch(nxt, jt + 1);                         // past the last tile: zeros / unused, harmless; issued between the MFMAs below
      const bf16_t* ks = cur;
      const bf16_t* vs = cur + TILE;
      // ---- S^T = K Q^T  (two blocks of 32 keys)
      f32x16_t st[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) st[jb][e] = 0.f;
#pragma unroll
        for (int s = 0; s < HD / 16; ++s)
          st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(ks, fo, jb, s), qf[s], st[jb], 0, 0, 0);
      }
      pipeline_reads_mfma_loads<16, 1, 8>();
      __builtin_amdgcn_sched_barrier(0);
      // ---- mask + tile maximum (register e of block jb is key j0 + 32 jb + 8 (e/4) + 4 hf + e%4).
      // Only tiles that straddle a limit of this wave evaluate the per-element predicate.
      float mx;
      const int rel = lim - j0 - 4 * hf;    // key offsets inside the tile are compile-time constants
      auto tile_max = [&](auto masked) {
        if (decltype(masked)::value) {
#pragma unroll
          for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              if (32 * jb + 8 * (e >> 2) + (e & 3) >= rel) st[jb][e] = -INFINITY;
            }
        }
        mx = st[0][0];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[jb][e]);
      };
      if (j0 + BJ > wave_lo) tile_max(std::true_type{}); else tile_max(std::false_type{});
      mx = half_pair_max(mx);
      // ---- online softmax for this lane's query.  The running reference m only moves when the
      // tile maximum exceeds it by more than 2^RESCALE_LOG2 in the exponent, so that most tiles
      // skip the rescaling of O; p then ranges up to 2^RESCALE_LOG2 instead of 1, which float
      // sums and bf16 probabilities (same relative precision) take without loss.
      const bool grow = (mx - m) * c2 > RESCALE_LOG2;      // also true for the first visible key (m = -inf)
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {         // wave-uniform
        const float m_new = grow ? mx : m;
        const float alpha = grow ? __builtin_amdgcn_exp2f((m - m_new) * c2) : 1.f;   // m = -inf: 0 (and O, l are 0)
        l *= alpha;
        m = m_new;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[i][e] *= alpha;
      }
      const float mc = (m == -INFINITY ? 0.f : m) * c2;
      float rs = 0.f;
      uint32_t pk[2][8];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[jb][e], c2, -mc));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[jb][e + 1], c2, -mc));
          rs += p0 + p1;
          pk[jb][e >> 1] = cvt_pk(p0, p1);
        }
      rs = half_pair_sum(rs);
      l += rs;
      // ---- O^T += V^T P^T ; step t of block jb uses S^T registers 8t .. 8t+7
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          union { uint32_t u[4]; bf16x8_t v; } pf;
#pragma unroll
          for (int i = 0; i < 4; ++i) pf.u[i] = pk[jb][4 * t + i];
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(vs, fo, 32 * jb + 16 * t, cb), pf.v, o[cb], 0, 0, 0);
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

  // ---- normalise and store: register e of block cb is channel 32 cb + 8 (e/4) + 4 hf + e%4
  // The rows go out through LDS (the stages are free: the last step, or the prologue, ended with a barrier).
  {
    const float inv = l > 0.f ? 1.f / l : 0.f;
    uint2 po[16];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd)
        po[4 * cb + qd] = make_uint2(cvt_pk(o[cb][4 * qd] * inv, o[cb][4 * qd + 1] * inv),
                                     cvt_pk(o[cb][4 * qd + 2] * inv, o[cb][4 * qd + 3] * inv));
    store_rows_via_lds(stage0 + wave * 32 * HD, po, lane, (bf16_t*)a.o + ((sv.q0 + qw0) * a.H + h) * HD, (int64_t)a.H * HD,
                       sv.S - qw0);
    if (q_ok && hf == 0)
      a.lse[sv.lse0 + h * sv.lse_hs + q] = l > 0.f ? m * a.scale + __logf(l) : -INFINITY;
  }
}

void launch_attn_fwd_bf16(const AttnArgs& a, hipStream_t s) {
  ProfScope ps("attn_fwd_bf16", s);
  dim3 grid(((a.S + fwd::BQ - 1) / fwd::BQ) * a.H * a.B);
  hipLaunchKernelGGL(attn_fwd_bf16_kernel, grid, dim3(256), 0, s, a);
}

}  // namespace beagle
