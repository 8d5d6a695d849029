// Decode-time draft step (section 4.1, KV-cache paragraph) for bf16, head
// width 128: M <= 64 draft queries per pass against L cached K/V rows, all
// visible.  The step is bound by HBM bandwidth (the K/V cache, Wq and Wo are
// each read once), so the kernels are shaped to put every CU's share of those
// bytes in flight at once (direct HBM -> LDS loads, whole chip resident in a
// single round); the matrix cores only keep arithmetic off the critical path.
//
//   (A) skinny_gemm   q_part[ks] = x * Wq[k-slice ks]        grid (N/64) x (K/512),
//                     two workgroups per CU, the whole chip resident at once; the
//                     64 KB tile is worked on in quarters as they land
//   (B) decode_attn   one workgroup per (head, key range, block of 32 queries);
//                     its 4 waves split each 128-key step by rows.  A lane owns
//                     one query (as in the training forward): online softmax per
//                     lane, P goes from the accumulator registers straight into
//                     the second MFMA.  q is the sum of (A)'s k-slices, split
//                     into a bf16 hi + lo pair so that scores (and the LSE) see
//                     q at ~16 bits.  Waves are merged in LDS; each range writes
//                     an unnormalised partial.
//   (C) combine       merges the key ranges, writes o (bf16) and the LSE; with up
//                     to 4 queries this runs in the prologue of (D) instead
//   (D) skinny_gemm   y_part[ks] = o * Wo[k-slice ks]
//   (E) sum_slices    y = sum_ks y_part[ks]  (bf16)
//
// With drafted states concatenated to the cache (appendix "Ablation Study", "concate" with the
// drafting tree) the rows at and past n_true are visible to a query only where
// its row of the tree bitmask has a bit; (B) applies it to the 32-key blocks
// that reach past n_true.  Appending up to 64 states to the cache runs (A) on
// Wk and Wv in one launch (z = 0, 1) and (E) into the cache rows.
//
// Partial results cross workgroups only at kernel boundaries: on this chip a
// device-scope fence inside a kernel writes back a whole L2 (the XCDs' L2s are
// not coherent with each other), which costs far more than a launch.  All sums
// run in a fixed order, so results are bitwise reproducible.
#include <type_traits>
#include "attn_tiles.h"

namespace beagle {
using namespace tiles;

namespace dec {
constexpr int MAXM = 64;               // queries per pass
constexpr int SG_N = 64;               // output columns per workgroup
constexpr int SG_K = 512;              // k rows per workgroup
constexpr int SG_KQ = SG_K / 4;        // k rows per quarter tile (32 per wave)
constexpr int KSTEP = 128;             // keys per attention step (32 per wave)
constexpr int TILE = KSTEP * HD;       // one K or V step tile
}  // namespace dec

// ---------------------------------------------------------------------------
// (A)/(C)  part[ks][m][n] = sum_{k in slice ks} x[m][k] * W[k][n]   (float)
//
// W tile in LDS: 512 k-rows of 64 columns (128 B, 8 chunks) in four quarters of
// 128 k-rows; chunk c of k-row k sits at chunk c ^ (((k >> 1) & 1) << 2), which
// makes the transpose reads (4 consecutive k-rows x 64 B) hit four different
// bank quarters.
// ---------------------------------------------------------------------------
//
// COMBINE: x is not read from memory.  It is the attention output of the M <= COMB_MAXM draft queries, merged here
// from the split-KV partials of (B) while the W tile is on its way: the workgroup's 512 k are the channels
// of 4 heads, each the (max, sum)-weighted mean of R key ranges; the result is rounded to bf16 as the
// stand-alone merge (C) does.  Workgroups of the first column block also write the LSE of their heads.
struct CombineArgs {
  const float* opart; const float* mlpart;   // [H][R][Mpad][128], [H][R][Mpad][2]
  float* lse; int lse_stride;                // [H][lse_stride]
  int Mpad, R;
  float scale;
};
// every projection workgroup repeats the merge of its 4 heads, one round trip to memory per two queries: beyond
// four queries the merge as a launch of its own is cheaper (measured at 8 and 10 queries)
constexpr int COMB_MAXM = 4, COMB_MAXR = 8;

typedef unsigned int xload_t __attribute__((ext_vector_type(4)));

template <bool COMBINE>
__global__ __launch_bounds__(256, 2) void skinny_gemm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ W,
                                                             float* __restrict__ part, int M, int N, int K, CombineArgs cb,
                                                             const bf16_t* __restrict__ W_z1, float* __restrict__ part_z1,
                                                             int x_chunked) {
  using namespace dec;
  if (blockIdx.z == 1) { W = W_z1; part = part_z1; }        // second weight matrix of the launch (same x)
  // The 64 KB tile as four quarters of 128 k-rows, one LDS variable each: requests land in the order they were
  // issued, so quarter c is complete when all but the 12 - 4c youngest have landed, and its transpose reads
  // (half-rate LDS instructions: 2 100 cycles for the whole tile with two workgroups per CU) run while the later
  // quarters are still on their way.  Only the last quarter's reads are exposed behind the data.
  __shared__ __attribute__((aligned(1024))) bf16_t wt0[SG_KQ * SG_N];
  __shared__ __attribute__((aligned(1024))) bf16_t wt1[SG_KQ * SG_N];
  __shared__ __attribute__((aligned(1024))) bf16_t wt2[SG_KQ * SG_N];
  __shared__ __attribute__((aligned(1024))) bf16_t wt3[SG_KQ * SG_N];
  __shared__ __attribute__((aligned(16))) bf16_t xs[COMBINE ? COMB_MAXM * SG_K : 8];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5;
  const int n0 = blockIdx.x * SG_N, ks = blockIdx.y, k0 = ks * SG_K;
  const int mblocks = (M + 31) / 32;

  // Loads whose values this wave needs first go first (a wave's loads return in order).
  // plain: x fragments (B operand): lane holds x[m][k0 + 128 c + 32 wave + 16 s2 + 8 hf .. +7] as xf[mb][2 c + s2]
  bf16x8_t xf[2][8];
  // COMBINE: item = (query m, head hh of the 4, float4 column c4); all R ranges of a thread's (up to two) items
  constexpr int NIT = COMB_MAXM * 4 * 32 / 256;
  float2 ml[COMBINE ? NIT : 1][COMB_MAXR];
  float4 ov[COMBINE ? NIT : 1][COMB_MAXR];
  if (!COMBINE) {
    // branch-free: rows past M and channels past K are asked for beyond the end of the descriptor and arrive as zeros
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)((int64_t)M * K * 2), 0x00020000);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
      for (int st = 0; st < 8; ++st) {
        const bf16x8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
        xf[mb][st] = z;
      }
      if (mb < mblocks) {
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          const int m = 32 * mb + (lane & 31), k = k0 + (st >> 1) * SG_KQ + wave * 32 + (st & 1) * 16 + 8 * hf;
          union { xload_t u; bf16x8_t v; } t;
          // x_chunked: x is stored [K / 8][M][8] -- the 32 rows of a fragment are 512 contiguous bytes, where the row-major
          // layout has 32 bytes of each of 32 rows (the range merge writes its output that way for this kernel)
          const int off = x_chunked ? ((k >> 3) * M + m) * 16 : (m * K + k) * 2;
          t.u = __builtin_amdgcn_raw_buffer_load_b128(xrs, (m < M && k < K) ? off : (int)0x80000000, 0, 0);
          xf[mb][st] = t.v;
        }
      }
    }
  } else {
    // unconditional loads from clamped indices (ranges past R repeat range 0, queries past M repeat the last one): a
    // select on a loaded value here would make the compiler wait for each load before it issues the next
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (256 * it < M * 128) {
        const int idx = tid + 256 * it;
        const int c4 = idx & 31, hh = (idx >> 5) & 3, m = min(idx >> 7, M - 1);
        const int h = k0 / HD + hh;
        const float* mlp = cb.mlpart + ((int64_t)h * cb.R * cb.Mpad + m) * 2;
        const float* ovp = cb.opart + ((int64_t)h * cb.R * cb.Mpad + m) * HD + 4 * c4;
#pragma unroll
        for (int r = 0; r < COMB_MAXR; ++r) {
          const int rr = (r < cb.R ? r : 0) * cb.Mpad;          // wave-uniform
          ml[it][r] = *(const float2*)(mlp + rr * 2);
          ov[it][r] = *(const float4*)(ovp + rr * HD);
        }
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // the whole tile is requested at once: 16 loads of 16 bytes per lane in flight
  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void*)W, 0, (int)((int64_t)K * N * 2), 0x00020000);
  auto request = [&](bf16_t* wq, int c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int q = tid + 256 * i, k = q >> 3, ch = (q & 7) ^ (((k >> 1) & 1) << 2);
      const int off = (int)(((int64_t)(k0 + c * SG_KQ + k) * N + n0 + 8 * ch) * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(wrs, (lds_void_ptr)(wq + (i * 4 + wave) * 512), 16, off, 0, 0, 0);
    }
  };
  request(wt0, 0); request(wt1, 1); request(wt2, 2); request(wt3, 3);
  __builtin_amdgcn_sched_barrier(0);

  float lsev[COMBINE ? NIT : 1];             // stored at the end: a store in flight would blur the count of landed requests
  if (COMBINE) {
    const float c2 = cb.scale * LOG2E;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int idx = tid + 256 * it;
      const int c4 = idx & 31, hh = (idx >> 5) & 3, m = idx >> 7;
      lsev[it] = 0.f;
      if (m < M) {
        float mr[COMB_MAXR];
        float mm = -INFINITY;
#pragma unroll
        for (int r = 0; r < COMB_MAXR; ++r) { mr[r] = r < cb.R ? ml[it][r].x : -INFINITY; mm = fmaxf(mm, mr[r]); }
        float4 acc = {0.f, 0.f, 0.f, 0.f};
        float lt = 0.f;
#pragma unroll
        for (int r = 0; r < COMB_MAXR; ++r) {                  // fixed order
          const float sc = mr[r] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mr[r] - mm) * c2);
          acc.x += ov[it][r].x * sc; acc.y += ov[it][r].y * sc; acc.z += ov[it][r].z * sc; acc.w += ov[it][r].w * sc;
          lt += ml[it][r].y * sc;
        }
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        uint2 v = {cvt_pk(acc.x * inv, acc.y * inv), cvt_pk(acc.z * inv, acc.w * inv)};
        *(uint2*)(xs + m * SG_K + hh * HD + 4 * c4) = v;
        lsev[it] = lt > 0.f ? mm * cb.scale + logf(lt) : -INFINITY;
      }
    }
  }

  f32x16_t acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  const int gi = lane >> 4, r16 = lane & 15;
  // one quarter: the wave's 32 k-rows of it; the number of query blocks is a compile-time constant of each copy so that
  // the eight transpose reads are issued together, ahead of the MFMAs
  auto quarter_mb = [&](const bf16_t* wq, int c, auto mbc) {
    constexpr int MB = decltype(mbc)::value;
    bf16x8_t wf[2][2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int kr = wave * 32 + s2 * 16 + 8 * (gi >> 1) + (r16 >> 2);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const int col = 32 * nb + 16 * (gi & 1) + 4 * (r16 & 3);
        const bf16_t* p0 = wq + kr * SG_N + ((((col >> 3) ^ (((kr >> 1) & 1) << 2)) << 3) | (col & 7));
        const bf16_t* p1 = wq + (kr + 4) * SG_N + ((((col >> 3) ^ ((((kr + 4) >> 1) & 1) << 2)) << 3) | (col & 7));
        union { struct { s16x4_t a, b; } s; bf16x8_t v; } u;
        u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
        u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p1);
        wf[s2][nb] = u.v;
      }
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s2][nb], xf[mb][2 * c + s2], acc[nb][mb], 0, 0, 0);
  };
  auto quarter = [&](const bf16_t* wq, int c) {
    if (mblocks == 1) quarter_mb(wq, c, std::integral_constant<int, 1>{});
    else quarter_mb(wq, c, std::integral_constant<int, 2>{});
  };

  wait_vmem_n<12>();
  lds_barrier();                            // quarter 0 (and the merged x) complete for every wave
  if (COMBINE) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const int m = lane & 31;
      bf16x8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
      xf[0][st] = m < M ? *(const bf16x8_t*)(xs + m * SG_K + (st >> 1) * SG_KQ + wave * 32 + (st & 1) * 16 + 8 * hf) : z;
      xf[1][st] = z;
    }
  }
  quarter(wt0, 0);
  wait_vmem_n<8>();
  lds_barrier();
  quarter(wt1, 1);
  wait_vmem_n<4>();
  lds_barrier();
  quarter(wt2, 2);
  wait_vmem_n<0>();
  lds_barrier();
  quarter(wt3, 3);
  // up to 32 queries the merge below uses quarters 0 and 2 only, which every wave has left behind at the last barrier
  if (mblocks > 1) lds_barrier();

  // merge the four waves' k-shares through LDS, one quarter per (column half nb, query block mb):
  // red[2 nb + mb][wave][m % 32][(n % 32 + 4 m) % 32] (the rotation spreads the per-row float4 writes over the banks)
  auto red = [&](int i) -> float* { return (float*)(i == 0 ? wt0 : i == 1 ? wt1 : i == 2 ? wt2 : wt3); };
  static_assert(4 * 32 * 32 * sizeof(float) <= sizeof(wt0), "merge buffer must fit in a quarter tile");
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
      if (mb < mblocks) {
        const int ml = lane & 31;
        if (32 * mb + ml < M) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nl = 8 * q + 4 * hf;
            float4 v = {acc[nb][mb][4 * q], acc[nb][mb][4 * q + 1], acc[nb][mb][4 * q + 2], acc[nb][mb][4 * q + 3]};
            *(float4*)(red(2 * nb + mb) + (wave * 32 + ml) * 32 + ((nl + 4 * ml) & 31)) = v;
          }
        }
      }
  __syncthreads();
  for (int i = tid; i < M * (SG_N / 4); i += 256) {
    const int m = i / (SG_N / 4), n = (i % (SG_N / 4)) * 4;
    const int ml = m & 31, nr = ((n & 31) + 4 * ml) & 31;
    const float* rp = red(2 * (n >> 5) + (m >> 5)) + ml * 32 + nr;
    float4 s = *(const float4*)rp;
#pragma unroll
    for (int wv = 1; wv < 4; ++wv) {
      const float4 t = *(const float4*)(rp + wv * 32 * 32);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    *(float4*)(part + ((int64_t)ks * M + m) * N + n0 + n) = s;
  }
  if (COMBINE && blockIdx.x == 0) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int idx = tid + 256 * it;
      const int c4 = idx & 31, hh = (idx >> 5) & 3, m = idx >> 7;
      if (m < M && c4 == 0) cb.lse[(int64_t)(k0 / HD + hh) * cb.lse_stride + m] = lsev[it];
    }
  }
}

// y[m][n] = sum_ks part[ks][m][n] (+ res[m][n])  -> bf16
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ part, bf16_t* __restrict__ y,
                                                         int64_t MN, int KS, const float* __restrict__ part_z1,
                                                         bf16_t* __restrict__ y_z1, const bf16_t* __restrict__ res) {
  // (all arguments at hand after one trip to the constant cache: placed where each is first used, they made three)
  asm volatile("" :: "s"(part), "s"(y), "s"(MN), "s"(KS), "s"(part_z1), "s"(y_z1), "s"(res));
  if (blockIdx.z == 1) { part = part_z1; y = y_z1; res = nullptr; }
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= MN) return;
  // eight slices (and the residual) are loaded before any is added (one round trip to memory, not eight or nine); the
  // order of the sum is fixed
  uint2 r = {0u, 0u};
  float4 s = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < KS; k0 += 8) {
    float4 t[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = *(const float4*)(part + (int64_t)min(k0 + k, KS - 1) * MN + i);
    if (k0 == 0 && res) r = *(const uint2*)(res + i);       // behind the first batch's requests, ahead of their use
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k0 + k < KS) { s.x += t[k].x; s.y += t[k].y; s.z += t[k].z; s.w += t[k].w; }
  }
  if (res) {                                  // residual connection of Eq. 1
    s.x += __uint_as_float(r.x << 16); s.y += __uint_as_float(r.x & 0xffff0000u);
    s.z += __uint_as_float(r.y << 16); s.w += __uint_as_float(r.y & 0xffff0000u);
  }
  uint2 v = {cvt_pk(s.x, s.y), cvt_pk(s.z, s.w)};
  *(uint2*)(y + i) = v;
}

// m[i] = silu(sum_ks upart[ks][i]) * sum_ks wpart[ks][i]  -> bf16   (gate of the feed-forward layer, Eq. 1)
__global__ __launch_bounds__(256) void sum_gate_kernel(const float* __restrict__ upart, const float* __restrict__ wpart,
                                                       bf16_t* __restrict__ m, int64_t MN, int KS) {
  asm volatile("" :: "s"(upart), "s"(wpart), "s"(m), "s"(MN), "s"(KS));
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= MN) return;
  float4 u = {0.f, 0.f, 0.f, 0.f}, w = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < KS; k0 += 8) {        // eight slices of each in flight at a time
    float4 a[8], b[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int64_t o = (int64_t)min(k0 + k, KS - 1) * MN + i;
      a[k] = *(const float4*)(upart + o); b[k] = *(const float4*)(wpart + o);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k0 + k < KS) {
        u.x += a[k].x; u.y += a[k].y; u.z += a[k].z; u.w += a[k].w;
        w.x += b[k].x; w.y += b[k].y; w.z += b[k].z; w.w += b[k].w;
      }
  }
  auto silu = [](float t) { return t / (1.f + expf(-t)); };
  uint2 v = {cvt_pk(silu(u.x) * w.x, silu(u.y) * w.y), cvt_pk(silu(u.z) * w.z, silu(u.w) * w.w)};
  *(uint2*)(m + i) = v;
}

// ---------------------------------------------------------------------------
// (D')  y[m][n] = sum_k a[m][k] * W[k][n]  (+ res[m][n]) for up to 16 rows, on a weight matrix that was packed for
// this kernel once per model load (pack_strips_kernel below).  A workgroup owns a strip of 16 output columns over the
// whole of K, so there are N / 16 workgroups (one per CU at N = 4096) without any k split: no partial sums in memory
// and no launch to add them up.  Its waves take the 128-k macro-steps of the strip in turn.
//
// Packed layout: the 16 columns x 128 k of (macro-step m, strip s) are one 4 KB block at ((m * N/16) + s) * 4 KB, in
// the order the lanes consume them: 16 bytes of lane l for MFMA j at (j * 64 + l) * 16, holding
// W[128 m + 32 j + 8 (l / 16) + e][16 s + l % 16], e = 0..7 (column n = lane % 16, k group lane / 16 of a 32-k
// instruction).  So every load instruction reads 1 KB contiguous, a macro-step's blocks of all strips are contiguous,
// and the workgroups sweep the matrix together front to back: measured with loads only, 90 MB stream in 15.8 us
// this way (5.7 TB/s, what a plain contiguous read gets), against 17.5 us with each strip's blocks contiguous
// and 21.3 us for 16 rows x 64 B per instruction on a transposed matrix.  ST_FLIGHT macro-steps per wave are in flight.
// The activations are small and come from L2.  A wave parks those of its own macro-steps in LDS (chunk c of row m
// at chunk c ^ m: conflict-free fragment reads), a chunk of ST_CH macro-steps at a time in two buffers: the first
// two chunks are requested before the first weights (requests complete in order: behind the weights they would
// arrive behind them, and the MFMAs of a macro-step could not start when its weights land), every later chunk one
// chunk ahead of its use, in front of the weight refills of that chunk.  The buffers are private to the wave, so
// the loop has no barrier; everything is ordinary loads and LDS traffic that the compiler counts by itself.
// Rows past M hold whatever LDS held: an MFMA output row depends on its own input row only, and rows past M
// are not stored.
//
// MODE 1 (one query): a is not read; it is the attention output merged here from the split-KV partials of (B), as
// in skinny_gemm_kernel<true>, each wave for the heads that are its macro-steps (at most ST_CH: K <= 4096);
// workgroup 0 writes the LSE.
// MODE 2 (feed-forward layer, Eq. 1): two weight matrices share the activations, and the strip's result is
// silu(a W) * (a W2): the gate needs no launch of its own.
// MODE 3 (cache append): two weight matrices share the activations, each with an output of its own (K and V rows).
// ---------------------------------------------------------------------------
namespace dec {
constexpr int ST_N = 16;                 // output columns per workgroup
constexpr int ST_FLIGHT = 4;             // weight macro-steps (4 KB) in flight per wave, over all matrices
constexpr int ST_ROUND = 4;              // macro-steps per unrolled round of the loop
constexpr int ST_MAXM = 16;              // rows per launch
}  // namespace dec
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

template <int MODE, bool ROWS16, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void strip_gemm_kernel(const bf16_t* __restrict__ a, const bf16_t* __restrict__ Wt,
                                                            const bf16_t* __restrict__ Wt2, void* __restrict__ yout,
                                                            bf16_t* __restrict__ yout2, const bf16_t* __restrict__ res,
                                                            int M, int N, int K, CombineArgs cb, int out_f32,
                                                            float norm_eps) {
  using namespace dec;
  asm volatile("" :: "s"(a), "s"(Wt), "s"(Wt2), "s"(yout), "s"(yout2), "s"(res), "s"(M), "s"(N), "s"(K), "s"(out_f32), "s"(norm_eps),
               "s"(cb.opart), "s"(cb.mlpart), "s"(cb.lse), "s"(cb.lse_stride), "s"(cb.Mpad), "s"(cb.R), "s"(cb.scale));
  constexpr int ROWS = ROWS16 ? 16 : 8;             // activation rows kept per macro-step
  constexpr int ST_CH = ROWS16 ? 2 : 4;             // macro-steps per activation chunk
  constexpr int LPS = ROWS / 4;                     // loads per macro-step (1 KB = 4 rows each)
  constexpr int NLD = ST_CH * LPS;                  // loads per chunk: 8
  constexpr int NW = MODE >= 2 ? 2 : 1;             // weight matrices
  constexpr int ST_RING = ST_FLIGHT / NW;           // ring slots per matrix
  constexpr int ABUF = WAVES * ST_CH * ROWS * 256;  // one activation buffer of all waves: 64 KB with eight
  static_assert(ST_ROUND % ST_CH == 0 && ST_ROUND % ST_RING == 0, "chunks and ring slots repeat with the round");
  __shared__ __attribute__((aligned(1024))) unsigned char abuf[2][ABUF];
  __shared__ __attribute__((aligned(16))) float red[NW][WAVES][16][16];
  __shared__ __attribute__((aligned(16))) float wsc[MODE == 1 ? WAVES : 1][64];
  __shared__ float winv[MODE == 1 ? WAVES : 1][8];
  __shared__ float ssw[WAVES][16];                  // RMSNorm: each wave's share of the rows' sums of squares
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = blockIdx.x * ST_N;
  const int S = K >> 7;                             // macro-steps; wave w takes s = w, w + 8, ...
  const int nst = (S - wave + WAVES - 1) / WAVES;
  const int nl = lane & 15, kg = lane >> 4;
  unsigned char* aw0 = abuf[0] + wave * (ST_CH * ROWS * 256);
  unsigned char* aw1 = abuf[1] + wave * (ST_CH * ROWS * 256);

  float lse_out = -INFINITY;
  f32x4_t acc[NW];
#pragma unroll
  for (int w = 0; w < NW; ++w) acc[w] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float ssl[LPS];                       // RMSNorm: this lane's share of its rows' sums of squares
#pragma unroll
  for (int g = 0; g < LPS; ++g) ssl[g] = 0.f;
  const bool rownorm = norm_eps >= 0.f;
  if (nst > 0) {                        // (a wave without a macro-step, K < 1024, only adds zeros below)
  // ---- activations.  Load q of chunk c covers rows 4 g + kg of step c ST_CH + i, (i, g) = divmod(q, LPS):
  // lane (kg, nl) reads chunk nl ^ row of its row and parks it at chunk nl, i.e. at lane * 16 of the 1 KB piece.
  const __amdgpu_buffer_rsrc_t ars = __builtin_amdgcn_make_buffer_rsrc((void*)a, 0, MODE == 1 ? 0 : (int)((int64_t)M * K * 2), 0x00020000);
  auto stage_issue = [&](xload_t (&av)[NLD], int c) {
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
      const int i = c * ST_CH + q / LPS, row = 4 * (q % LPS) + kg;
      av[q] = __builtin_amdgcn_raw_buffer_load_b128(
          ars, (i < nst && row < M) ? (row * K + (wave + WAVES * i) * 128 + 8 * (nl ^ row)) * 2 : (int)0x80000000, 0, 0);
    }
  };
  // RMSNorm of the activation rows (norm_eps >= 0; Eq. 1's block normalises each sublayer's input): the gain is folded
  // into the packed weights and the row factor 1 / sqrt(mean(a^2) + eps) is applied to the finished sums, so all that is
  // needed here is the rows' sums of squares, gathered while the rows pass through registers on their way to LDS.
  // Load q of a chunk holds 8 values of row 4 (q % LPS) + kg; rows and steps past the end arrive as zeros.
  auto stage_park = [&](const xload_t (&av)[NLD], unsigned char* buf) {
#pragma unroll
    for (int q = 0; q < NLD; ++q) *(xload_t*)(buf + ((q / LPS) * ROWS + 4 * (q % LPS)) * 256 + lane * 16) = av[q];
    if (rownorm) {
#pragma unroll
      for (int q = 0; q < NLD; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = __uint_as_float(av[q][e] << 16), hi = __uint_as_float(av[q][e] & 0xffff0000u);
          ssl[q % LPS] += lo * lo + hi * hi;
        }
    }
  };
  xload_t av0[MODE == 1 ? 1 : NLD], av1[MODE == 1 ? 1 : NLD];
  float2 mlv = {-INFINITY, 0.f};
  float4 ov[MODE == 1 ? 2 : 1][COMB_MAXR];
  if constexpr (MODE != 1) {
    stage_issue(av0, 0);
    stage_issue(av1, 1);
  } else {
    // (max, sum) of head slot lane / 8, range lane % 8; then the partial outputs: item j = head slot 2 j + lane / 32,
    // float4 column lane % 32, all ranges (ranges past R repeat range 0 with weight 0; slots past the wave's last
    // repeat the last head: loads stay unconditional)
    const int hl = lane >> 3, r = lane & 7;
    if (hl < nst && r < cb.R)
      mlv = *(const float2*)(cb.mlpart + ((int64_t)((wave + WAVES * hl) * cb.R + r) * cb.Mpad) * 2);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int h2 = min(wave + WAVES * (2 * j + (lane >> 5)), S - 1);
#pragma unroll
      for (int rr = 0; rr < COMB_MAXR; ++rr)
        ov[j][rr] = *(const float4*)(cb.opart + ((int64_t)(h2 * cb.R + (rr < cb.R ? rr : 0)) * cb.Mpad) * HD + 4 * (lane & 31));
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- the first ST_RING macro-steps of weights (one matrix at K = 4096: all of them)
  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void*)Wt, 0, (int)((int64_t)N * K * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t wrs2 = __builtin_amdgcn_make_buffer_rsrc((void*)(MODE >= 2 ? Wt2 : Wt), 0, (int)((int64_t)N * K * 2), 0x00020000);
  const int wbase = blockIdx.x * 4096 + lane * 16;          // this strip's block of macro-step 0, this lane's 16 bytes
  const int wstep = (N / ST_N) * 4096;                      // from one macro-step's blocks to the next's
  union frag_t { xload_t u; bf16x8_t v; };
  frag_t bw[NW][ST_RING][4];
  auto load_b = [&](int u, int i) {
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        bw[w][u][j].u = __builtin_amdgcn_raw_buffer_load_b128(w == 0 ? wrs : wrs2, i < nst ? wbase + (wave + WAVES * i) * wstep + j * 1024 : (int)0x80000000, 0, 0);
  };
#pragma unroll
  for (int u = 0; u < ST_RING; ++u) load_b(u, u);
  __builtin_amdgcn_sched_barrier(0);

  if constexpr (MODE == 1) {
    const int hl = lane >> 3;
    const float c2 = cb.scale * LOG2E;
    float mm = mlv.x;
    mm = fmaxf(mm, __shfl_xor(mm, 1)); mm = fmaxf(mm, __shfl_xor(mm, 2)); mm = fmaxf(mm, __shfl_xor(mm, 4));
    const float sc = mlv.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mlv.x - mm) * c2);
    float lt = mlv.y * sc;
    lt += __shfl_xor(lt, 1); lt += __shfl_xor(lt, 2); lt += __shfl_xor(lt, 4);
    wsc[wave][lane] = sc;
    if ((lane & 7) == 0) winv[wave][hl] = lt > 0.f ? 1.f / lt : 0.f;
    lse_out = lt > 0.f ? mm * cb.scale + logf(lt) : -INFINITY;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int hl2 = 2 * j + (lane >> 5), c4 = lane & 31;
      uint2 v = {0u, 0u};                                      // slots past the wave's last head: zeros, not stale LDS
      if (hl2 < nst) {
        const float4 s0 = *(const float4*)&wsc[wave][hl2 * 8], s1 = *(const float4*)&wsc[wave][hl2 * 8 + 4];
        const float w[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        const float inv = winv[wave][hl2];
        float4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int rr = 0; rr < COMB_MAXR; ++rr) {               // fixed order
          t.x += ov[j][rr].x * w[rr]; t.y += ov[j][rr].y * w[rr]; t.z += ov[j][rr].z * w[rr]; t.w += ov[j][rr].w * w[rr];
        }
        v = uint2{cvt_pk(t.x * inv, t.y * inv), cvt_pk(t.z * inv, t.w * inv)};
      }
      *(uint2*)(aw0 + hl2 * ROWS * 256 + (c4 >> 1) * 16 + (c4 & 1) * 8) = v;        // row 0: chunk c at chunk c
    }
  } else {
    stage_park(av0, aw0);
    stage_park(av1, aw1);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- macro-steps, ST_ROUND to an unrolled round: activation fragments from the chunk's buffer, weights from the ring, the
  // slot's refill behind its MFMAs.  At a chunk's first step the chunk after the next is requested (in front of this
  // chunk's refills), at its last step it is parked in the buffer the chunk leaves behind.  No branches inside a
  // round: past the wave's last macro-step weights and activations are asked for beyond their descriptors' ends and
  // arrive as zeros, so every path holds the same number of requests in flight.
  const int mr = nl & (ROWS - 1);
  auto step = [&](int u, const unsigned char* buf, int slot) {
    frag_t af[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) af[j].u = *(const xload_t*)(buf + (slot * ROWS + mr) * 256 + (((4 * j + kg) ^ mr) & 15) * 16);
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[j].v, bw[w][u][j].v, acc[w], 0, 0, 0);
  };
  if (ST_RING == ST_ROUND && nst <= ST_RING) {      // the ring holds every macro-step: nothing to request any more
#pragma unroll
    for (int u = 0; u < ST_RING; ++u) step(u, (u / ST_CH) & 1 ? aw1 : aw0, u % ST_CH);
  } else if constexpr (MODE != 1) {
    int i0 = 0;
    do {
#pragma unroll
      for (int u = 0; u < ST_ROUND; ++u) {
        const int c = (i0 + u) / ST_CH;                        // chunk of this step; its buffer is c & 1
        unsigned char* buf = (c & 1) ? aw1 : aw0;
        if (u % ST_CH == 0) stage_issue(av0, c + 2);
        step(u % ST_RING, buf, u % ST_CH);
        load_b(u % ST_RING, i0 + u + ST_RING);
        if (u % ST_CH == ST_CH - 1) stage_park(av0, buf);
      }
      i0 += ST_ROUND;
    } while (i0 < nst);
  }
  }

  // ---- the waves' k shares, added in wave order; output row 4 kg + e, column nl
#pragma unroll
  for (int w = 0; w < NW; ++w)
#pragma unroll
    for (int e = 0; e < 4; ++e) red[w][wave][4 * kg + e][nl] = acc[w][e];
  if (MODE != 1 && rownorm) {
    // a row's 16 chunk lanes (same kg) add up, then the waves do below
#pragma unroll
    for (int g = 0; g < LPS; ++g) {
      float t = ssl[g];
      t += __shfl_xor(t, 1); t += __shfl_xor(t, 2); t += __shfl_xor(t, 4); t += __shfl_xor(t, 8);
      if (nl == 0) ssw[wave][4 * g + kg] = t;
    }
    if (ROWS == 8 && lane < 8) ssw[wave][8 + lane] = 0.f;
  }
  __syncthreads();
  if (tid < M * 16) {
    const int m = tid >> 4, n = tid & 15;
    float v = red[0][0][m][n];
#pragma unroll
    for (int wv = 1; wv < WAVES; ++wv) v += red[0][wv][m][n];
    float rn = 1.f;
    if (MODE != 1 && rownorm) {
      float ss = ssw[0][m];
#pragma unroll
      for (int wv = 1; wv < WAVES; ++wv) ss += ssw[wv][m];
      rn = 1.f / sqrtf(ss / (float)K + norm_eps);
      v *= rn;
    }
    const int64_t o = (int64_t)m * N + n0 + n;
    if constexpr (MODE >= 2) {
      float g = red[NW - 1][0][m][n];
#pragma unroll
      for (int wv = 1; wv < WAVES; ++wv) g += red[NW - 1][wv][m][n];
      if (MODE == 2) v = v / (1.f + expf(-v)) * (g * rn);      // silu(gate) * up
      else yout2[o] = (bf16_t)(cvt_pk(g * rn, 0.f) & 0xffffu); // the second matrix has its own output
    }
    if (res) v += __uint_as_float((uint32_t)res[o] << 16);
    if (out_f32) ((float*)yout)[o] = v;                       // the queries: the attention kernel wants them unrounded
    else ((bf16_t*)yout)[o] = (bf16_t)(cvt_pk(v, 0.f) & 0xffffu);
  }
  if (MODE == 1 && blockIdx.x == 0 && (lane & 7) == 0 && (lane >> 3) < nst)
    cb.lse[(int64_t)(wave + WAVES * (lane >> 3)) * cb.lse_stride] = lse_out;
}

// The one-time re-layout of a weight matrix W [K][N] (row-major) for strip_gemm_kernel: one thread per 16 bytes of
// the packed matrix (layout above).  K % 128 == 0, N % 16 == 0.
// With a gain vector g [K] the packed matrix is diag(g) W (each product rounded to bf16): the gain of an RMSNorm in front
// of the projection, so that the projection can take the un-normalised rows.
__global__ __launch_bounds__(256) void pack_strips_kernel(const bf16_t* __restrict__ in, bf16_t* __restrict__ out, int K, int N,
                                                          const bf16_t* __restrict__ gain) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;          // 16-byte piece of the output
  if (t >= (int64_t)K * N / 8) return;
  const int lane = (int)(t & 63), j = (int)((t >> 6) & 3);
  const int64_t blk = t >> 8;                                          // (m, s) = divmod(blk, N / 16)
  const int ns = N / 16, m = (int)(blk / ns), sidx = (int)(blk % ns);
  const int k0 = 128 * m + 32 * j + 8 * (lane >> 4), n = 16 * sidx + (lane & 15);
  bf16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] = in[(int64_t)(k0 + e) * N + n];
    if (gain) v[e] = (bf16_t)(cvt_pk(__uint_as_float((uint32_t)v[e] << 16) * __uint_as_float((uint32_t)gain[k0 + e] << 16), 0.f) & 0xffffu);
  }
  uint4 o = {(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16),
             (uint32_t)v[4] | ((uint32_t)v[5] << 16), (uint32_t)v[6] | ((uint32_t)v[7] << 16)};
  *(uint4*)(out + t * 8) = o;
}
void launch_pack_strips_bf16(const void* in, void* out, int32_t K, int32_t N, const void* gain, hipStream_t s) {
  const int64_t pieces = (int64_t)K * N / 8;
  hipLaunchKernelGGL(pack_strips_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, (const bf16_t*)in, (bf16_t*)out, K, N,
                     (const bf16_t*)gain);
}

// ---------------------------------------------------------------------------
// (B) split-KV attention: per (head, key range) partials
// ---------------------------------------------------------------------------
struct DecAttnArgs {
  const float* qpart; int KSq;            // [KSq][M][H*128]
  const bf16_t* kc; const bf16_t* vc;     // [L][G][128]
  float* opart; float* mlpart;            // [H][R][Mpad][128], [H][R][Mpad][2]
  int M, Mpad, L, H, G, R, range;
  float scale;
  // draft tree (nullptr: all rows visible): rows >= n_true are visible to query m iff bit (row - n_true) of
  // tree[m * tree_words ...] is set
  const uint32_t* tree; int n_true, tree_words;
  // rotary embedding of the queries: (cos, sin) of channel pair c of query m at rope_tab[m * 64 + c], or nullptr
  const float2* rope_tab;
};

// (cos, sin) of the rotary angles of M queries, evaluated in double: query m stands at pos[m] (or pos0), channel
// pair c < 64 turns by position * base^(-2c/128).
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* pos, int pos0, int M, float base, float2* tab) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M * 64) return;
  const int m = i >> 6, c = i & 63;
  double sn, cs;
  sincos((double)(pos ? pos[m] : pos0) * exp2(-2.0 * c / 128.0 * log2((double)base)), &sn, &cs);
  tab[i] = make_float2((float)cs, (float)sn);
}

// LDS reads with the address split into a register and a compile-time byte offset (at most 65 535): one address
// register serves every stage, plane and 16-row step that a fragment kind is read from.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
template <int OFF> __device__ __forceinline__ void lds_read_b128(xload_t& d, uint32_t addr) {
  static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF));
}
template <int OFF> __device__ __forceinline__ void lds_read_tr16_b64(u32x2_t& d, uint32_t addr) {
  static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF));
}
template <int V> struct int_c { static constexpr int value = V; };
template <int I, int N, class F> __device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) { f(int_c<I>{}); static_for<I + 1, N>(f); }
}

// One workgroup per (head, key range, block of 32 NQB queries): grid (H, R, ceil(M / (32 NQB))).
// NQB = 1 (up to 32 queries): the four waves split each 128-key step by rows, 32 keys each.  A wave requests, reads
// and refills only its own 32 rows of the two stages, so the step loop has no barrier; a stage half (the wave's K
// rows, then its V rows) is refilled for the step after next as soon as its fragments sit in registers, i.e. BEFORE
// the step's arithmetic: with both stages landed and nothing requested, HBM would idle for as long as a step
// computes (measured: 3 us of the kernel's 16).
// NQB = 2 (33 .. 64 queries): the same split of a step by rows; every wave works its 32 keys against both blocks of
// 32 queries, so K and V fragments are read from LDS once for the two blocks, no wave reads another's rows and the
// loop is as free of barriers as with one block.  (Waves 0, 1 on the first block and waves 2, 3 on the second, each
// with 64 keys of a step, was the earlier shape: stages shared between waves, hence a barrier per step with the
// refill issued only behind it -- 4 400 cycles of arithmetic and 2 700 of request issue per step, one after the other.)
template <int NQB>
__global__ __launch_bounds__(256, 1) void decode_attn_kernel(DecAttnArgs a) {
  using namespace dec;
  // two stages of one K and one V step tile each: tile t (0: K, 1: V) of stage i at (2 t + i) * TILE, so that the
  // two stages of a tile kind are 32 KB apart (within the offset field of an LDS read)
  __shared__ __attribute__((aligned(1024))) bf16_t kvt[4 * TILE];
  auto tile_of = [&](int si, int t) { return kvt + (2 * t + si) * TILE; };
  // q as bf16 planes of 32 queries: plane b = hi part of block b, plane NQB + b = its lo part.  With two blocks that
  // makes 160 KB with the stages: the merge's small arrays live in the planes, which are dead after the prologue.
  __shared__ __attribute__((aligned(1024))) bf16_t qbuf[2 * NQB * 32 * HD];
  typedef float ml_t[NQB][2][32];
  typedef float sc_t[NQB][32];
  ml_t* const s_ml = (ml_t*)qbuf;                                       // [wave]: running max, sum of its queries
  sc_t* const s_sc = (sc_t*)((float*)qbuf + 4 * NQB * 2 * 32);          // [wave]: merge weight of a wave's partial
  ml_t& s_mm = *(ml_t*)((float*)qbuf + 4 * NQB * 3 * 32);               // merged max, sum per block
  static_assert((4 * NQB * 3 * 32 + NQB * 2 * 32) * sizeof(float) <= sizeof(qbuf), "merge arrays must fit in the q planes");
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5, ql = lane & 31;
  const int h = blockIdx.x, r = blockIdx.y;
  const int m0 = 32 * NQB * blockIdx.z;                      // first query of the workgroup
  const int mtot = min(32 * NQB, a.M - m0);                  // its queries
  // every field at hand after one trip to the constant cache (the compiler otherwise fetches them where they are first
  // used, two dependent trips before the first K/V request); no division for the common one head per group
  asm volatile("" :: "s"(a.qpart), "s"(a.KSq), "s"(a.kc), "s"(a.vc), "s"(a.opart), "s"(a.mlpart), "s"(a.M), "s"(a.Mpad), "s"(a.L),
               "s"(a.H), "s"(a.G), "s"(a.R), "s"(a.range), "s"(a.scale), "s"(a.tree), "s"(a.n_true), "s"(a.tree_words),
               "s"(a.rope_tab));
  const int g = a.H == a.G ? h : h / (a.H / a.G);
  const int HDt = a.H * HD;
  const int j_begin = r * a.range, j_end = min(j_begin + a.range, a.L);
  const int nsteps = j_end > j_begin ? (j_end - j_begin + KSTEP - 1) / KSTEP : 0;

  const int64_t kvs = (int64_t)a.G * HD;
  const __amdgpu_buffer_rsrc_t krs = rows_rsrc(a.kc + (int64_t)g * HD, j_end, kvs);   // rows >= j_end read as zero
  const __amdgpu_buffer_rsrc_t vrs = rows_rsrc(a.vc + (int64_t)g * HD, j_end, kvs);
  // the same step requested by waves 1 .. 3 only: request n of the 64 (32 per tile, 64 chunks of 16 bytes each) is wave 1 + n % 3's
  auto fetch3 = [&](int si, int step) {
    const int row0 = j_begin + step * KSTEP;
#pragma unroll
    for (int n0 = 0; n0 < 66; n0 += 3) {
      const int n = n0 + wave - 1;
      if (n < 64) {
        const int q = 64 * (n & 31) + lane, rr = q >> 4, c = (q & 15) ^ swz(rr);
        const int off = (int)(((int64_t)(row0 + rr) * kvs + 8 * c) * 2);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(n < 32 ? krs : vrs, (lds_void_ptr)(tile_of(si, n >> 5) + (n & 31) * 512), 16, off, 0, 0, 0);
      }
    }
  };
  // this wave's own 32 rows of a step's K (t = 0) or V (t = 1) tile: 8 requests, no branch (rows past the range read as zero)
  auto fetch_own_half = [&](int si, int step, int t) {
    const int row0 = j_begin + step * KSTEP;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int q = 512 * wave + 64 * i + lane, rr = q >> 4, c = (q & 15) ^ swz(rr);
      const int off = (int)(((int64_t)(row0 + rr) * kvs + 8 * c) * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(t ? vrs : krs, (lds_void_ptr)(tile_of(si, t) + (8 * wave + i) * 512), 16, off, 0, 0, 0);
    }
  };
  auto fetch_own = [&](int si, int step) { fetch_own_half(si, step, 0); fetch_own_half(si, step, 1); };
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) float* lds_float_ptr;
  typedef __attribute__((address_space(3))) bf16_t* lds_bf16_ptr;
  const float4 zero4 = {0.f, 0.f, 0.f, 0.f};

  // ---- q = sum of the projection's k-slices (fixed order).  The workgroup sums a block once and leaves it in LDS
  // as a bf16 hi + lo pair (hi = bf16(q), lo = bf16(q - hi): scores, and the LSE, see q at ~16 bits), rows of 128
  // channels = 16 chunks of 16 bytes, chunk c of row m at chunk position c ^ (m % 16) so that the per-query
  // fragment reads spread over the banks; then every lane picks up its B-operand fragments.  A thread of a summing
  // wave holds four float4 of the block: (query idx >> 5, channels 4 (idx & 31) ..) with idx = tid + 64 qwaves i.
  // Loads of slices, rows and waves that do not take part are asked for past the end of the buffer, i.e. arrive as
  // zeros: no branches around loads, so that the compiler can count the requests between a load and its use (a
  // wave's loads return in order).
  const int64_t slice = (int64_t)a.M * HDt;                             // floats per k-slice
  const __amdgpu_buffer_rsrc_t qrs =
      __builtin_amdgcn_make_buffer_rsrc((void*)a.qpart, 0, (int)(a.KSq * slice * 4), 0x00020000);
  const int oob = 0x7fffff00;
  auto q_issue = [&](int qb, int mrows, int qwaves, int k0, u32x4_t (&t)[4][8]) {
    const int mb = m0 + 32 * qb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + 64 * qwaves * i, m = idx >> 5, c4 = idx & 31;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int off = (int)((((int64_t)(k0 + k) * a.M + mb + m) * HDt + h * HD + 4 * c4) * 4);
        t[i][k] = __builtin_amdgcn_raw_buffer_load_b128(qrs, (wave < qwaves && m < mrows && k0 + k < a.KSq) ? off : oob, 0, 0);
      }
    }
  };
  auto q_add = [&](const u32x4_t (&t)[4][8], float4 (&acc)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        acc[i].x += __uint_as_float(t[i][k][0]); acc[i].y += __uint_as_float(t[i][k][1]);
        acc[i].z += __uint_as_float(t[i][k][2]); acc[i].w += __uint_as_float(t[i][k][3]);
      }
  };
  // slices past the first eight (model widths above 4096), and the rotary embedding: this thread's four channels of
  // query m pair with the four that lane ^ 16 holds (float4 slot c4 ^ 16 of the same query)
  auto q_finish = [&](int qb, int mrows, int qwaves, float4 (&acc)[4]) {
    for (int k0 = 8; k0 < a.KSq; k0 += 8) {
      u32x4_t t[4][8];
      q_issue(qb, mrows, qwaves, k0, t);
      q_add(t, acc);
    }
    if (a.rope_tab) {
      const int mb = m0 + 32 * qb;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = tid + 64 * qwaves * i, m = min(idx >> 5, mrows - 1), c4 = idx & 15;
        const float4* tp = (const float4*)(a.rope_tab + (int64_t)(mb + m) * 64 + 4 * c4);
        const float4 cs0 = tp[0], cs1 = tp[1];                 // (cos, sin) of pairs 4 c4 .. 4 c4 + 3
        const bool upper = (tid & 16) != 0;                    // channels 64 .. 127: x2 of the pair
        const float4 own = acc[i];
        float4 oth;
        oth.x = __shfl_xor(own.x, 16, 64); oth.y = __shfl_xor(own.y, 16, 64);
        oth.z = __shfl_xor(own.z, 16, 64); oth.w = __shfl_xor(own.w, 16, 64);
        // x1' = x1 cos - x2 sin ; x2' = x2 cos + x1 sin
        const float sg = upper ? 1.f : -1.f;
        acc[i].x = own.x * cs0.x + sg * oth.x * cs0.y;
        acc[i].y = own.y * cs0.z + sg * oth.y * cs0.w;
        acc[i].z = own.z * cs1.x + sg * oth.z * cs1.y;
        acc[i].w = own.w * cs1.z + sg * oth.w * cs1.w;
      }
    }
  };
  // hi / lo halves (8 bytes each) of four channels of row m
  auto q_split = [&](const float4& v, uint2& hi, uint2& lo) {
    const float f[4] = {v.x, v.y, v.z, v.w};
    float rem[4];
    uint32_t h16[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const __bf16 hb = (__bf16)f[i];
      rem[i] = f[i] - (float)hb;
      h16[i] = (uint32_t)__builtin_bit_cast(unsigned short, hb);
    }
    hi = make_uint2(h16[0] | (h16[1] << 16), h16[2] | (h16[3] << 16));
    lo = make_uint2(cvt_pk(rem[0], rem[1]), cvt_pk(rem[2], rem[3]));
  };
  auto q_slot = [&](int m, int c4) { return m * HD + ((((c4 >> 1) ^ (m & 15)) << 3) | ((c4 & 1) << 2)); };   // element offset
  // a summing wave's four float4 into the block buffer, with explicit LDS instructions: HBM -> LDS requests are in
  // flight, and for LDS accesses it can see the compiler would wait for all of them
  auto q_store = [&](int qb, int qwaves, const float4 (&acc)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + 64 * qwaves * i, m = idx >> 5, c4 = idx & 31;
      uint2 hi, lo;
      q_split(acc[i], hi, lo);
      const u32x2_t vh = {hi.x, hi.y}, vl = {lo.x, lo.y};
      asm volatile("ds_write_b64 %0, %1" : : "v"((lds_bf16_ptr)(qbuf + qb * 32 * HD + q_slot(m, c4))), "v"(vh) : "memory");
      asm volatile("ds_write_b64 %0, %1" : : "v"((lds_bf16_ptr)(qbuf + (NQB + qb) * 32 * HD + q_slot(m, c4))), "v"(vl) : "memory");
    }
  };
  // B-operand fragments of a plane (explicit ds_read, see above): channels 16 s + 8 hf .. + 7 of query ql
  typedef union { u32x4_t u; bf16x8_t v; } qfrag_t;
  auto issue_frags = [&](int plane, qfrag_t (&f)[8]) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
      asm volatile("ds_read_b128 %0, %1" : "=v"(f[s].u) : "v"((lds_bf16_ptr)(qbuf + plane * 32 * HD + ql * HD + (((2 * s + hf) ^ (ql & 15)) << 3))));
  };
  auto tie_frags = [&](qfrag_t (&f)[8]) {     // after the wait: nothing that uses the values may be scheduled above it
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(f[s].u));
  };
  auto read_frags = [&](int plane, bf16x8_t (&out)[8]) {
    qfrag_t f[8];
    issue_frags(plane, f);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    tie_frags(f);
#pragma unroll
    for (int s = 0; s < 8; ++s) out[s] = f[s].v;
  };

  // this lane's fragments of q (one block; with two they stay in their LDS planes and are read again in every step)
  bf16x8_t qh[1][8], qlo[1][8];
  bool shared_first_steps = false;                           // steps 0 and 1 requested across waves (barrier before step 1)
  if (NQB == 1 && mtot <= 8) {
    // Up to 8 queries: wave 0 alone sums (one round trip for its 32 loads) while waves 1 .. 3 request the first
    // two K/V steps at once, wave 0's share included: the 64 requests of a step go round waves 1, 2, 3 (22, 21 and
    // 21 of them).  q is there long before the first step has landed.
    shared_first_steps = true;
    if (wave == 0) {
      u32x4_t t[4][8];
      float4 acc[4] = {zero4, zero4, zero4, zero4};
      q_issue(0, mtot, 1, 0, t);
      q_add(t, acc);
      q_finish(0, mtot, 1, acc);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = tid + 64 * i, m = idx >> 5, c4 = idx & 31;
        uint2 hi, lo;
        q_split(acc[i], hi, lo);
        *(uint2*)(qbuf + q_slot(m, c4)) = hi;
        *(uint2*)(qbuf + 32 * HD + q_slot(m, c4)) = lo;
      }
    } else {
      // rows 8 .. 31 hold no query: zeros in both planes (16 bytes per thread and step)
      for (int idx = tid - 64; idx < 2 * 24 * 16; idx += 192) {
        const int pl = idx / (24 * 16), rest = idx % (24 * 16);
        *(uint4*)(qbuf + pl * 32 * HD + (8 + rest / 16) * HD + (rest % 16) * 8) = make_uint4(0, 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (wave > 0) {
      if (nsteps > 0) fetch3(0, 0);
      if (nsteps > 1) fetch3(1, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (nsteps > 0 && wave > 0) {
      // all but the wave's requests of the second step have landed
      if (nsteps == 1) wait_vmem(); else if (wave == 1) wait_vmem_n<22>(); else wait_vmem_n<21>();
    }
    lds_barrier();                                             // first K/V step landed; q sum visible
    read_frags(0, qh[0]);
    read_frags(1, qlo[0]);
  } else if (NQB == 1) {
    // 9 .. 32 queries: two or four waves sum.  Every wave requests its own rows of step 0, then its q slices, then
    // its rows of step 1 -- the K/V stream starts with the kernel, and q (loads return in order) is complete when
    // step 0 has landed, which the arithmetic has to wait for anyway.
    const int qwaves = mtot <= 16 ? 2 : 4;
    u32x4_t t[4][8];
    float4 acc[4] = {zero4, zero4, zero4, zero4};
    fetch_own(0, 0);
    q_issue(0, mtot, qwaves, 0, t);
    fetch_own(1, 1);
    __builtin_amdgcn_sched_barrier(0);
    wait_vmem_n<16>();                                         // all but step 1's requests
    q_add(t, acc);
    if (wave < qwaves) {
      q_finish(0, mtot, qwaves, acc);
      q_store(0, qwaves, acc);
    } else {
      // rows 16 .. 31 hold no query (two summing waves cover 16): zeros in both planes, from the other two waves
      for (int idx = tid - 64 * qwaves; idx < 2 * 16 * 16; idx += 256 - 64 * qwaves) {
        const int pl = idx >> 8, rest = idx & 255;
        const u32x4_t z = {0u, 0u, 0u, 0u};
        asm volatile("ds_write_b128 %0, %1" : : "v"((lds_bf16_ptr)(qbuf + pl * 32 * HD + (16 + (rest >> 4)) * HD + (rest & 15) * 8)), "v"(z) : "memory");
      }
    }
    lds_barrier();                                             // q visible
    read_frags(0, qh[0]);
    read_frags(1, qlo[0]);
  } else {
    // 33 .. 64 queries, all four waves sum both blocks: own rows of step 0, block 0's slices, own rows of step 1,
    // block 1's slices -- the last of these only issue as the oldest requests retire (a wave holds at most 63), which
    // is when step 0 lands, and are back soon after step 1.
    u32x4_t t0[4][8], t1[4][8];
    float4 acc[4] = {zero4, zero4, zero4, zero4};
    fetch_own(0, 0);
    q_issue(0, 32, 4, 0, t0);
    fetch_own(1, 1);
    q_issue(1, mtot - 32, 4, 0, t1);                           // rows past the last query: zeros
    __builtin_amdgcn_sched_barrier(0);
    wait_vmem_n<48>();                                         // step 0 and block 0's slices
    q_add(t0, acc);
    q_finish(0, 32, 4, acc);
    q_store(0, 4, acc);
    wait_vmem();
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = zero4;
    q_add(t1, acc);
    q_finish(1, mtot - 32, 4, acc);
    q_store(NQB - 1, 4, acc);
    lds_barrier();                                             // both blocks visible
  }
  const float c2 = a.scale * LOG2E;
  const FragOffs fo = make_frag_offs(lane);

  f32x16_t o[NQB][4];
  float mrun[NQB], lrun[NQB];
#pragma unroll
  for (int b = 0; b < NQB; ++b) {
    mrun[b] = -INFINITY; lrun[b] = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[b][i][e] = 0.f;
  }

  bool o_zero = true;                                        // wave-uniform: nothing accumulated into O yet
  // Per-lane LDS byte addresses of the three fragment kinds; stages, planes and 16-row steps add compile-time offsets.
  const uint32_t kvt_a = (uint32_t)(uintptr_t)(lds_bf16_ptr)kvt, qbuf_a = (uint32_t)(uintptr_t)(lds_bf16_ptr)qbuf;
  uint32_t ka[8], va[4][2], qa[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    ka[s] = kvt_a + 2 * (wave * 32 * HD + fo.row[s]);                          // K tile of stage 0, this wave's rows
    qa[s] = qbuf_a + 2 * (ql * HD + (((2 * s + hf) ^ (ql & 15)) << 3));        // plane 0
  }
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int i = 0; i < 2; ++i) va[cb][i] = kvt_a + 2 * (2 * TILE + wave * 32 * HD + fo.tr[cb][i]);   // V tile of stage 0
  constexpr int STAGE_B = TILE * 2, PLANE_B = 32 * HD * 2, TSTEP_B = 16 * HD * 2;   // byte distances

  // One 128-key step on stage SI: this wave's 32 rows of the step tiles against its query blocks; `refill` requests
  // the same rows of step + 2 into the stage as soon as their fragments have been read.
  auto step_compute = [&](auto stage_c, int step, bool refill) {
    constexpr int SI = decltype(stage_c)::value;
    const int kb = wave;                                       // 32-row block of the step tiles
    const int jw = j_begin + step * KSTEP + 32 * kb;           // its first key
    if (jw < j_end) {
      // Explicit ds_read instructions (same addresses as row_frag / tr_frag): for LDS reads it can see, the compiler
      // waits until no HBM -> LDS request is in flight at all, and the refills would never overlap the arithmetic.
      union { xload_t u; bf16x8_t v; } kf[8];
      union { struct { u32x2_t x, y; } s; bf16x8_t v; } vf[2][4];
      auto issue_v = [&]() {
        static_for<0, 2>([&](auto t_) {
          constexpr int t = decltype(t_)::value;
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) {
            lds_read_tr16_b64<SI * STAGE_B + t * TSTEP_B>(vf[t][cb].s.x, va[cb][0]);
            lds_read_tr16_b64<SI * STAGE_B + t * TSTEP_B>(vf[t][cb].s.y, va[cb][1]);
          }
        });
      };
#pragma unroll
      for (int s = 0; s < 8; ++s) lds_read_b128<SI * STAGE_B>(kf[s].u, ka[s]);
      f32x16_t st[NQB];
#pragma unroll
      for (int b = 0; b < NQB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) st[b][e] = 0.f;
      // LDS reads return in order and the counter holds at most 15: at most 15 of 24 still out means the first 9
      // are there, the 8 K fragments among them
      if constexpr (NQB == 1) {
        issue_v();
        asm volatile("s_waitcnt lgkmcnt(15)" ::: "memory");
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(kf[s].u));
        // two independent accumulation chains (hi and lo part of q) halve the dependent-MFMA latency
        f32x16_t st2;
#pragma unroll
        for (int e = 0; e < 16; ++e) st2[e] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          st[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, qh[0][s], st[0], 0, 0, 0);
          st2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, qlo[0][s], st2, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) st[0][e] += st2[e];
      } else {
        // One chain per block, hi parts first.  q's fragments come from their LDS planes in every step (the two output
        // accumulators fill the accumulation registers, and 128 more registers of fragments did not survive register
        // allocation): the lo fragments land during the hi parts' MFMAs, the V fragments during the lo parts'.
        qfrag_t qf[NQB][8], ql_[NQB][8];
        static_for<0, NQB>([&](auto b_) {
          constexpr int b = decltype(b_)::value;
#pragma unroll
          for (int s = 0; s < 8; ++s) lds_read_b128<b * PLANE_B>(qf[b][s].u, qa[s]);
        });
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(kf[s].u));
#pragma unroll
        for (int b = 0; b < NQB; ++b) tie_frags(qf[b]);
        static_for<0, NQB>([&](auto b_) {
          constexpr int b = decltype(b_)::value;
#pragma unroll
          for (int s = 0; s < 8; ++s) lds_read_b128<(NQB + b) * PLANE_B>(ql_[b][s].u, qa[s]);
        });
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
          for (int b = 0; b < NQB; ++b) st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, qf[b][s].v, st[b], 0, 0, 0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < NQB; ++b) tie_frags(ql_[b]);
        issue_v();
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
          for (int b = 0; b < NQB; ++b) st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, ql_[b][s].v, st[b], 0, 0, 0);
      }
      // The wave's K rows are in registers: refill them.  Behind the MFMAs in program order: while every CU
      // streams, a request waits in the issue stage for a slot in the memory pipeline (about 170 cycles each),
      // and the matrix pipe works through the scores meanwhile.
      __builtin_amdgcn_sched_barrier(0);
      if (refill) fetch_own_half(SI, step + 2, 0);
      __builtin_amdgcn_sched_barrier(0);
      uint32_t pk[NQB][8];
#pragma unroll
      for (int b = 0; b < NQB; ++b) {
        f32x16_t& sb = st[b];
        if (jw + 32 > j_end) {
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (jw + 8 * (e >> 2) + 4 * hf + (e & 3) >= j_end) sb[e] = -INFINITY;
        }
        if (a.tree != nullptr && jw + 32 > a.n_true) {
          // drafted rows: bit i of `vis` says whether this lane's query sees key jw + i (true rows: yes)
          const int off = jw - a.n_true;                       // tree bit of key jw; negative inside the true rows
          const int w0 = off >> 5, sh = off & 31;              // floor division: -1 for the straddling block
          const uint32_t* row = a.tree + (int64_t)(m0 + 32 * b + ql) * a.tree_words;
          const bool real = 32 * b + ql < mtot;
          const uint32_t lo = w0 < 0 ? 0xffffffffu : (real && w0 < a.tree_words ? row[w0] : 0u);
          const uint32_t hi = real && w0 + 1 < a.tree_words ? row[w0 + 1] : 0u;
          const uint32_t vis = (uint32_t)((((uint64_t)hi << 32) | lo) >> sh);
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (!((vis >> (8 * (e >> 2) + 4 * hf + (e & 3))) & 1u)) sb[e] = -INFINITY;
        }
        float mx = sb[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sb[e]);
        mx = half_pair_max(mx);
        // the running reference moves only when the block maximum exceeds it by more than 2^8 in the
        // exponent (p then ranges up to 2^8: harmless for float sums and bf16 probabilities), so that most
        // steps skip the rescaling of O
        const bool grow = (mx - mrun[b]) * c2 > 8.f;           // also true at the first step (reference -inf)
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {          // wave-uniform
          const float m_new = grow ? mx : mrun[b];             // finite: the block holds at least one real key
          const float alpha = grow ? __builtin_amdgcn_exp2f((mrun[b] - m_new) * c2) : 1.f;
          lrun[b] *= alpha;
          mrun[b] = m_new;
          if (!o_zero) {                                       // (the first block a wave works on always grows: O is still 0)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int e = 0; e < 16; ++e) o[b][i][e] *= alpha;
          }
        }
        const float mc = (mrun[b] == -INFINITY ? 0.f : mrun[b]) * c2;   // nothing visible so far: p = exp2(-inf) = 0
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(sb[e] * c2 - mc);
          const float p1 = __builtin_amdgcn_exp2f(sb[e + 1] * c2 - mc);
          rs += p0 + p1;
          pk[b][e >> 1] = cvt_pk(p0, p1);
        }
        rs = half_pair_sum(rs);
        lrun[b] += rs;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the V fragments
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) asm volatile("" : "+v"(vf[t][cb].s.x), "+v"(vf[t][cb].s.y));
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int b = 0; b < NQB; ++b) {
          union { uint32_t u[4]; bf16x8_t v; } pf;
#pragma unroll
          for (int i = 0; i < 4; ++i) pf.u[i] = pk[b][4 * t + i];
#pragma unroll
          for (int cb = 0; cb < 4; ++cb)
            o[b][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][cb].v, pf.v, o[b][cb], 0, 0, 0);
        }
      o_zero = false;
      __builtin_amdgcn_sched_barrier(0);
      if (refill) fetch_own_half(SI, step + 2, 1);             // ... and the wave's V rows, behind the P V MFMAs
      __builtin_amdgcn_sched_barrier(0);
    } else if (refill) {
      fetch_own(SI, step + 2);                                 // keeps every wave's request count the same
    }
  };

  // Two stages.  Before step s the wave's rows of s must have landed: the only younger requests are those of
  // step s + 1 (issued during step s - 1).  With up to 8 queries the first two steps were requested across
  // waves, hence the one barrier before step 1.
#pragma unroll 1
  for (int step = 0; step < nsteps; step += 2) {
    if (step > 0) {
      if (step + 1 < nsteps) wait_vmem_n<16>(); else wait_vmem();
    }
    step_compute(int_c<0>{}, step, step + 2 < nsteps);
    if (step + 1 < nsteps) {
      if (step + 2 < nsteps) wait_vmem_n<16>(); else wait_vmem();
      if (shared_first_steps && step == 0) lds_barrier();
      step_compute(int_c<1>{}, step + 1, step + 3 < nsteps);
    }
  }

  // ---- merge the waves' partials of each query block (fixed order) and write this key range's partial.
  // Buffer of block b (64 KB of the stages): [4 waves][32 queries][128 channels] floats; a float4 of query q sits 4 q floats
  // further round its row, so that neither the per-query writes nor the per-channel reads conflict.
  __syncthreads();
  static_assert(NQB * 4 * 32 * HD * sizeof(float) <= sizeof(kvt), "the merge buffers must fit in the stages");
  const int64_t pbase = ((int64_t)h * a.R + r) * a.Mpad + m0;
#pragma unroll
  for (int b = 0; b < NQB; ++b) {
    float* ob = (float*)kvt + b * 4 * 32 * HD;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int c = 32 * cb + 8 * e4 + 4 * hf;
        const float4 v = {o[b][cb][4 * e4], o[b][cb][4 * e4 + 1], o[b][cb][4 * e4 + 2], o[b][cb][4 * e4 + 3]};
        *(float4*)(ob + (wave * 32 + ql) * HD + ((c + 4 * ql) & (HD - 1))) = v;
      }
    if (hf == 0) { s_ml[wave][b][0][ql] = mrun[b]; s_ml[wave][b][1][ql] = lrun[b]; }
  }
  __syncthreads();
  if (tid < 32 * NQB) {                                       // per query: the merged (max, sum) and each wave's weight
    const int qb = tid >> 5, q = tid & 31;
    float mm = -INFINITY;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) mm = fmaxf(mm, s_ml[wv][qb][0][q]);
    float lt = 0.f;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      const float mw = s_ml[wv][qb][0][q];
      const float sc = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mw - mm) * c2);
      s_sc[wv][qb][q] = sc;
      lt += s_ml[wv][qb][1][q] * sc;
    }
    s_mm[qb][0][q] = mm; s_mm[qb][1][q] = lt;
  }
  __syncthreads();
  for (int i = tid; i < mtot * 32; i += 256) {                 // padding rows are never read
    const int c4 = i & 31, qq = i >> 5, qb = qq >> 5, q = qq & 31;
    const float* ob = (const float*)kvt + qb * 4 * 32 * HD;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      const float sc = s_sc[wv][qb][q];
      const float4 v = *(const float4*)(ob + (wv * 32 + q) * HD + ((4 * c4 + 4 * q) & (HD - 1)));
      acc.x += v.x * sc; acc.y += v.y * sc; acc.z += v.z * sc; acc.w += v.w * sc;
    }
    *(float4*)(a.opart + (pbase + qq) * HD + 4 * c4) = acc;
    if (c4 == 0) { a.mlpart[(pbase + qq) * 2] = s_mm[qb][0][q]; a.mlpart[(pbase + qq) * 2 + 1] = s_mm[qb][1][q]; }
  }
}

// ---- (C) merge the key ranges (fixed order): o (bf16) and LSE ------------------
__global__ __launch_bounds__(128) void decode_combine_kernel(const float* __restrict__ opart, const float* __restrict__ mlpart,
                                                             bf16_t* __restrict__ o, float* __restrict__ lse,
                                                             int lse_stride, int Mpad, int H, int R, float scale,
                                                             int chunked_rows) {
  asm volatile("" :: "s"(opart), "s"(mlpart), "s"(o), "s"(lse), "s"(lse_stride), "s"(Mpad), "s"(H), "s"(R), "s"(scale), "s"(chunked_rows));
  const int m = blockIdx.x, h = blockIdx.y, c = threadIdx.x;
  const float c2 = scale * LOG2E;
  const int64_t p0 = (int64_t)h * R * Mpad + m;              // range s sits at p0 + s * Mpad
  // Eight ranges are loaded at a time before any is used, maxima, sums and outputs together: with up to eight ranges
  // the whole merge is one round trip to memory (the kernel is nothing but round trips: a pass over the maxima first
  // and the rest behind it cost a second one).  A batch that reaches past the last range repeats it, which changes
  // neither the maximum nor (weight 0) the sums.
  float ms[8], ls[8], ov[8];
  auto load_batch = [&](int s0) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int64_t pb = p0 + (int64_t)min(s0 + k, R - 1) * Mpad;
      ms[k] = mlpart[pb * 2]; ls[k] = mlpart[pb * 2 + 1]; ov[k] = opart[pb * HD + c];
    }
  };
  load_batch(0);
  float mm = -INFINITY;
#pragma unroll
  for (int k = 0; k < 8; ++k) mm = fmaxf(mm, ms[k]);
  for (int s0 = 8; s0 < R; s0 += 8) {                          // more than eight ranges: the remaining maxima first
    float t[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = mlpart[(p0 + (int64_t)min(s0 + k, R - 1) * Mpad) * 2];
#pragma unroll
    for (int k = 0; k < 8; ++k) mm = fmaxf(mm, t[k]);
  }
  float acc = 0.f, lt = 0.f;
  for (int s0 = 0; s0 < R; s0 += 8) {
    if (s0 > 0) load_batch(s0);
#pragma unroll
    for (int k = 0; k < 8; ++k) {                              // fixed order
      const float sc = (s0 + k < R && ms[k] > -INFINITY) ? __builtin_amdgcn_exp2f((ms[k] - mm) * c2) : 0.f;
      acc += ov[k] * sc;
      lt += ls[k] * sc;
    }
  }
  // chunked_rows (the split-k projection reads the merged rows): o as [H d / 8][rows][8], rows = chunked_rows; else [rows][H d]
  const int64_t oi = chunked_rows ? ((int64_t)((h * HD + c) >> 3) * chunked_rows + m) * 8 + (c & 7) : ((int64_t)m * H + h) * HD + c;
  o[oi] = f32_to_bf16(lt > 0.f ? acc / lt : 0.f);
  if (c == 0) lse[(int64_t)h * lse_stride + m] = lt > 0.f ? mm * scale + logf(lt) : -INFINITY;
}

// Plain streaming read of `bytes` bytes (16 bytes per lane, eight loads in flight per lane): the reference point for
// what the memory system delivers to a kernel that does nothing but read.
__global__ __launch_bounds__(256) void read_probe_kernel(const uint4* __restrict__ p, int64_t n16, uint32_t* __restrict__ sink) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  uint32_t acc = 0;
  for (int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x; i0 < n16; i0 += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int64_t i = i0 + u * stride;
      v[u] = i < n16 ? p[i] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) *sink = acc;          // keeps the loads alive; practically never taken
}
void launch_read_probe(const void* buf, int64_t bytes, int wgs, uint32_t* sink, hipStream_t s) {
  hipLaunchKernelGGL(read_probe_kernel, dim3(wgs), dim3(256), 0, s, (const uint4*)buf, bytes / 16, sink);
}

// Many one-wave workgroups, so that nearly every compute unit runs one: each writes the shader-cycle counter and the
// constant-rate (100 MHz) device clock, read back to back, into the slot of the place it finds itself on (XCD number
// and the shader-engine / array / compute-unit bits of the hardware id).  Cycle counters of different places are not
// aligned, so differences are only taken within a slot.
__global__ void clock_probe_kernel(uint64_t* __restrict__ out) {
  if (threadIdx.x == 0) {
    uint32_t xcc, hw;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    const uint32_t slot = ((xcc & 7u) << 8) | ((hw >> 8) & 0xffu);
    const uint64_t cyc = __builtin_readcyclecounter();
    const uint64_t real = __builtin_amdgcn_s_memrealtime();
    out[2 * slot] = cyc;
    out[2 * slot + 1] = real;
  }
}
void launch_clock_probe(uint64_t* out, hipStream_t s) {
  hipLaunchKernelGGL(clock_probe_kernel, dim3(1024), dim3(64), 0, s, out);
}

// ---- host side ----------------------------------------------------------------
namespace {
struct DecLayout {
  int KSq, KSo, R, range, Mpad;
  size_t qpart, opart, mlpart, o, ypart, ropetab, total;
};
size_t up256(size_t v) { return (v + 255) / 256 * 256; }
DecLayout dec_layout(int M, int L, int H, int d, int D) {
  DecLayout w;
  const int Mp = M < dec::MAXM ? M : dec::MAXM;             // queries per pass
  const int64_t HDt = (int64_t)H * d;
  w.KSq = (D + dec::SG_K - 1) / dec::SG_K;
  w.KSo = (int)((HDt + dec::SG_K - 1) / dec::SG_K);
  // key ranges per head: about one workgroup per CU over all heads, whole 128-key steps
  int R = 256 / H;
  if (R < 1) R = 1;
  const int max_r = (L + dec::KSTEP - 1) / dec::KSTEP;
  if (R > max_r) R = max_r;
  w.range = ((L + R - 1) / R + dec::KSTEP - 1) / dec::KSTEP * dec::KSTEP;
  w.R = (L + w.range - 1) / w.range;
  w.Mpad = (Mp + 31) / 32 * 32;
  size_t o = 0;
  w.qpart = o; o += up256((size_t)w.KSq * Mp * HDt * 4);
  w.opart = o; o += up256((size_t)H * w.R * w.Mpad * tiles::HD * 4);
  w.mlpart = o; o += up256((size_t)H * w.R * w.Mpad * 2 * 4);
  w.o = o; o += up256((size_t)Mp * HDt * 2);
  w.ypart = o; o += up256((size_t)w.KSo * Mp * D * 4);
  w.ropetab = o; o += up256((size_t)M * 64 * sizeof(float2));
  w.total = o;
  return w;
}
}  // namespace

// strip_gemm_kernel serves [M, K] x [N, K]^T when its rows fit one launch and its strips tile N
bool strip_gemm_fits(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || M > dec::ST_MAXM || N % dec::ST_N || K % 128 || K < 128) return false;
  return (int64_t)N * K * 2 < ((int64_t)1 << 31) && (int64_t)M * K * 2 < ((int64_t)1 << 31);
}
// y = a W (+ res) on packed W; with wt2: y = silu(a W) * (a W2); with merge: a is merged from the attention partials (M = 1)
void launch_strip_gemm(const bf16_t* a, const bf16_t* wt, const bf16_t* wt2, void* y, bf16_t* y2, const bf16_t* res, int M,
                       int N, int K, const CombineArgs* merge, bool out_f32, float norm_eps, hipStream_t s) {
  using namespace dec;
  const dim3 grid(N / ST_N);
  const CombineArgs cb = merge ? *merge : CombineArgs{};
  const int f = out_f32 ? 1 : 0;
  // one matrix: eight waves, one workgroup per CU (N / 16 is about the number of CUs for the attention's projections);
  // the feed-forward pair has several strips per CU: four waves and two workgroups per CU, so that one's start and
  // final reduction hide behind the other's stream; the K/V pair of the cache append (y2 given) is as wide as one matrix
#define STRIP_ARGS a, wt, wt2, y, y2, res, M, N, K, cb, f, norm_eps
  if (merge) hipLaunchKernelGGL((strip_gemm_kernel<1, false, 8>), grid, dim3(512), 0, s, STRIP_ARGS);
  else if (wt2 && y2 && M <= 8) hipLaunchKernelGGL((strip_gemm_kernel<3, false, 8>), grid, dim3(512), 0, s, STRIP_ARGS);
  else if (wt2 && y2) hipLaunchKernelGGL((strip_gemm_kernel<3, true, 8>), grid, dim3(512), 0, s, STRIP_ARGS);
  else if (wt2 && M <= 8) hipLaunchKernelGGL((strip_gemm_kernel<2, false, 4>), grid, dim3(256), 0, s, STRIP_ARGS);
  else if (wt2) hipLaunchKernelGGL((strip_gemm_kernel<2, true, 4>), grid, dim3(256), 0, s, STRIP_ARGS);
  else if (M <= 8) hipLaunchKernelGGL((strip_gemm_kernel<0, false, 8>), grid, dim3(512), 0, s, STRIP_ARGS);
  else hipLaunchKernelGGL((strip_gemm_kernel<0, true, 8>), grid, dim3(512), 0, s, STRIP_ARGS);
#undef STRIP_ARGS
}

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
  float2* ropetab = a.rope ? (float2*)(base + w.ropetab) : nullptr;
  if (a.rope) {
    ProfScope ps("draft_rope_table", s);
    hipLaunchKernelGGL(rope_table_kernel, dim3((a.M * 64 + 255) / 256), dim3(256), 0, s, a.rope_pos, a.L, a.M,
                       a.rope_base, ropetab);
  }
  for (int m0 = 0; m0 < a.M; m0 += MAXM) {
    const int Mp = a.M - m0 < MAXM ? a.M - m0 : MAXM;
    const bf16_t* x = (const bf16_t*)a.x + (int64_t)m0 * a.D;
    if (a.wq_pk) {                    // packed Wq: the whole of k in one strip, so q arrives as a single slice
      ProfScope ps("draft_proj_q", s);
      launch_strip_gemm(x, (const bf16_t*)a.wq_pk, nullptr, qpart, nullptr, nullptr, Mp, HDt, a.D, nullptr, true, a.x_norm_eps, s);
    } else {
      ProfScope ps("draft_proj_q", s);
      hipLaunchKernelGGL(skinny_gemm_kernel<false>, dim3(HDt / SG_N, w.KSq), dim3(256), 0, s, x, (const bf16_t*)a.wq, qpart,
                         Mp, HDt, a.D, CombineArgs{}, (const bf16_t*)nullptr, (float*)nullptr, 0);
    }
    {
      DecAttnArgs t;
      t.qpart = qpart; t.KSq = a.wq_pk ? 1 : w.KSq; t.kc = (const bf16_t*)a.kc; t.vc = (const bf16_t*)a.vc;
      t.opart = opart; t.mlpart = mlpart;
      t.M = Mp; t.Mpad = w.Mpad; t.L = a.L; t.H = a.H; t.G = a.G; t.R = w.R; t.range = w.range;
      t.scale = a.scale;
      t.tree = a.tree ? a.tree + (int64_t)m0 * a.tree_words : nullptr; t.n_true = a.n_true; t.tree_words = a.tree_words;
      t.rope_tab = ropetab ? ropetab + (int64_t)m0 * 64 : nullptr;
      ProfScope ps("draft_attn", s);
      if (Mp > 32) hipLaunchKernelGGL(decode_attn_kernel<2>, dim3(a.H, w.R, (Mp + 63) / 64), dim3(256), 0, s, t);
      else hipLaunchKernelGGL(decode_attn_kernel<1>, dim3(a.H, w.R, 1), dim3(256), 0, s, t);
    }
    if (a.wo_pk) {
      // out-projection on the transposed weights: no k split, so no partial sums and no launch to add them
      CombineArgs cb;
      cb.opart = opart; cb.mlpart = mlpart; cb.lse = a.lse + m0; cb.lse_stride = a.M; cb.Mpad = w.Mpad; cb.R = w.R;
      cb.scale = a.scale;
      bf16_t* yo = (bf16_t*)a.y + (int64_t)m0 * a.D;
      const bf16_t* yr = a.y_res ? (const bf16_t*)a.y_res + (int64_t)m0 * a.D : (const bf16_t*)nullptr;
      if (Mp == 1 && w.R <= COMB_MAXR && HDt / HD <= 32) {
        ProfScope ps("draft_proj_out", s);
        launch_strip_gemm(nullptr, (const bf16_t*)a.wo_pk, nullptr, yo, nullptr, yr, Mp, a.D, HDt, &cb, false, -1.f, s);
      } else {
        {
          ProfScope ps("draft_combine", s);
          hipLaunchKernelGGL(decode_combine_kernel, dim3(Mp, a.H), dim3(128), 0, s, opart, mlpart, o, a.lse + m0, a.M,
                             w.Mpad, a.H, w.R, a.scale, 0);
        }
        ProfScope ps("draft_proj_out", s);
        launch_strip_gemm(o, (const bf16_t*)a.wo_pk, nullptr, yo, nullptr, yr, Mp, a.D, HDt, nullptr, false, -1.f, s);
      }
      continue;
    }
    if (Mp <= COMB_MAXM && w.R <= COMB_MAXR && HDt % SG_K == 0) {
      // few queries: the merge of the key ranges rides in the projection's prologue
      CombineArgs cb;
      cb.opart = opart; cb.mlpart = mlpart; cb.lse = a.lse + m0; cb.lse_stride = a.M; cb.Mpad = w.Mpad; cb.R = w.R;
      cb.scale = a.scale;
      ProfScope ps("draft_proj_out", s);
      hipLaunchKernelGGL(skinny_gemm_kernel<true>, dim3(a.D / SG_N, w.KSo), dim3(256), 0, s, (const bf16_t*)nullptr,
                         (const bf16_t*)a.wo, ypart, Mp, a.D, HDt, cb, (const bf16_t*)nullptr, (float*)nullptr, 0);
    } else {
      {
        ProfScope ps("draft_combine", s);
        hipLaunchKernelGGL(decode_combine_kernel, dim3(Mp, a.H), dim3(128), 0, s, opart, mlpart, o, a.lse + m0, a.M,
                           w.Mpad, a.H, w.R, a.scale, Mp);
      }
      ProfScope ps("draft_proj_out", s);
      hipLaunchKernelGGL(skinny_gemm_kernel<false>, dim3(a.D / SG_N, w.KSo), dim3(256), 0, s, (const bf16_t*)o,
                         (const bf16_t*)a.wo, ypart, Mp, a.D, HDt, CombineArgs{}, (const bf16_t*)nullptr, (float*)nullptr, 1);
    }
    {
      ProfScope ps("draft_sum_out", s);
      const int64_t MN = (int64_t)Mp * a.D;
      hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((MN / 4 + 255) / 256)), dim3(256), 0, s, ypart,
                         (bf16_t*)a.y + (int64_t)m0 * a.D, MN, w.KSo, (const float*)nullptr, (bf16_t*)nullptr,
                         a.y_res ? (const bf16_t*)a.y_res + (int64_t)m0 * a.D : (const bf16_t*)nullptr);
    }
  }
}

// ---- K and V rows of up to 64 new states, written into the cache rows at kdst / vdst ([n][N] contiguous):
// the two projections share one split-k launch (z = 0: Wk, z = 1: Wv) and one slice sum.
size_t kv_append_bf16_ws_bytes(int32_t n, int32_t N, int32_t K) {
  const int KS = (K + dec::SG_K - 1) / dec::SG_K;
  return 2 * up256((size_t)KS * n * N * 4);
}
bool kv_append_bf16_fits(int32_t n, int32_t N, int32_t K) {
  return n >= 1 && n <= dec::MAXM && N % dec::SG_N == 0 && K % 8 == 0 && (int64_t)K * N * 2 < ((int64_t)1 << 31);
}
void launch_kv_append_bf16(const void* x, const void* wk, const void* wv, void* kdst, void* vdst, int32_t n, int32_t N,
                           int32_t K, void* ws, hipStream_t s) {
  using namespace dec;
  const int KS = (K + SG_K - 1) / SG_K;
  float* kpart = (float*)ws;
  float* vpart = (float*)((char*)ws + up256((size_t)KS * n * N * 4));
  {
    ProfScope ps("kv_append_proj", s);
    hipLaunchKernelGGL(skinny_gemm_kernel<false>, dim3(N / SG_N, KS, 2), dim3(256), 0, s, (const bf16_t*)x,
                       (const bf16_t*)wk, kpart, n, N, K, CombineArgs{}, (const bf16_t*)wv, vpart, 0);
  }
  {
    ProfScope ps("kv_append_sum", s);
    const int64_t MN = (int64_t)n * N;
    hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((MN / 4 + 255) / 256), 1, 2), dim3(256), 0, s, kpart,
                       (bf16_t*)kdst, MN, KS, (const float*)vpart, (bf16_t*)vdst, (const bf16_t*)nullptr);
  }
}


// ---- feed-forward layer of the draft block for a handful of rows (decode time): HBM-bound on the three weight
// matrices, so the same split-k streaming projection: [z W_gate, z W_up] in one launch (z = 0 / 1), the gate fused
// into their slice sum, then m W_down with the residual added in its slice sum.  Rows are taken MAXM at a time.
namespace {
struct MlpLayout { int KSg, KSd; size_t upart, wpart, m, dpart, total; };
MlpLayout mlp_layout(int M, int D, int F) {
  MlpLayout w;
  const int Mp = M < dec::MAXM ? M : dec::MAXM;
  w.KSg = (D + dec::SG_K - 1) / dec::SG_K;
  w.KSd = (F + dec::SG_K - 1) / dec::SG_K;
  size_t o = 0;
  w.upart = o; o += up256((size_t)w.KSg * Mp * F * 4);
  w.wpart = o; o += up256((size_t)w.KSg * Mp * F * 4);
  w.m = o; o += up256((size_t)Mp * F * 2);
  w.dpart = o; o += up256((size_t)w.KSd * Mp * D * 4);
  w.total = o;
  return w;
}
}  // namespace

size_t block_mlp_bf16_ws_bytes(int32_t M, int32_t D, int32_t F) { return mlp_layout(M, D, F).total; }
bool block_mlp_bf16_fits(int32_t D, int32_t F) {
  return D % dec::SG_N == 0 && F % dec::SG_N == 0 && (int64_t)D * F * 2 < ((int64_t)1 << 31);
}
void launch_block_mlp_bf16(const void* z, const void* w_gate, const void* w_up, const void* w_down, const void* y_res,
                           void* h, int32_t M, int32_t D, int32_t F, void* ws, hipStream_t s) {
  using namespace dec;
  const MlpLayout w = mlp_layout(M, D, F);
  char* base = (char*)ws;
  float* upart = (float*)(base + w.upart);
  float* wpart = (float*)(base + w.wpart);
  bf16_t* mbuf = (bf16_t*)(base + w.m);
  float* dpart = (float*)(base + w.dpart);
  for (int m0 = 0; m0 < M; m0 += MAXM) {
    const int Mp = M - m0 < MAXM ? M - m0 : MAXM;
    const bf16_t* zr = (const bf16_t*)z + (int64_t)m0 * D;
    {
      ProfScope ps("draft_mlp_gate_up", s);
      hipLaunchKernelGGL(skinny_gemm_kernel<false>, dim3(F / SG_N, w.KSg, 2), dim3(256), 0, s, zr, (const bf16_t*)w_gate,
                         upart, Mp, F, D, CombineArgs{}, (const bf16_t*)w_up, wpart, 0);
    }
    {
      ProfScope ps("draft_mlp_gate", s);
      const int64_t MN = (int64_t)Mp * F;
      hipLaunchKernelGGL(sum_gate_kernel, dim3((unsigned)((MN / 4 + 255) / 256)), dim3(256), 0, s, upart, wpart, mbuf, MN, w.KSg);
    }
    {
      ProfScope ps("draft_mlp_down", s);
      hipLaunchKernelGGL(skinny_gemm_kernel<false>, dim3(D / SG_N, w.KSd), dim3(256), 0, s, (const bf16_t*)mbuf,
                         (const bf16_t*)w_down, dpart, Mp, D, F, CombineArgs{}, (const bf16_t*)nullptr, (float*)nullptr, 0);
    }
    {
      ProfScope ps("draft_mlp_sum", s);
      const int64_t MN = (int64_t)Mp * D;
      hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((MN / 4 + 255) / 256)), dim3(256), 0, s, dpart,
                         (bf16_t*)h + (int64_t)m0 * D, MN, w.KSd, (const float*)nullptr, (bf16_t*)nullptr,
                         (const bf16_t*)y_res + (int64_t)m0 * D);
    }
  }
}

// K and V rows of up to 16 new states on packed Wk, Wv (norm_eps >= 0: the RMSNorm in front of them, gain folded into
// the matrices): one strip launch, no workspace
void launch_kv_append_strip_bf16(const void* x, const void* wk_pk, const void* wv_pk, void* kdst, void* vdst, int32_t n,
                                 int32_t N, int32_t K, float norm_eps, hipStream_t s) {
  ProfScope ps("kv_append_proj", s);
  launch_strip_gemm((const bf16_t*)x, (const bf16_t*)wk_pk, (const bf16_t*)wv_pk, kdst, (bf16_t*)vdst, nullptr, n, N, K, nullptr,
                    false, norm_eps, s);
}

void launch_block_mlp_strip_bf16(const void* z, const void* w_gate_pk, const void* w_up_pk, const void* w_down_pk,
                                 const void* y_res, void* h, int32_t M, int32_t D, int32_t F, float z_norm_eps, void* ws,
                                 hipStream_t s) {
  bf16_t* mbuf = (bf16_t*)ws;
  {
    ProfScope ps("draft_mlp_gate_up", s);
    launch_strip_gemm((const bf16_t*)z, (const bf16_t*)w_gate_pk, (const bf16_t*)w_up_pk, mbuf, nullptr, nullptr, M, F, D, nullptr, false, z_norm_eps, s);
  }
  {
    ProfScope ps("draft_mlp_down", s);
    launch_strip_gemm(mbuf, (const bf16_t*)w_down_pk, nullptr, (bf16_t*)h, nullptr, (const bf16_t*)y_res, M, D, F, nullptr, false, -1.f, s);
  }
}

}  // namespace beagle
