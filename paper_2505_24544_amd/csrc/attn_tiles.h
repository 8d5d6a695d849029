// LDS tile helpers shared by the bf16 attention kernels (head width 128).
//
// A tile holds rows of 128 channels (256 B, 16 chunks of 16 B) in HBM order.
// Chunk c of row r is stored at chunk position c ^ swz(r), swz(r) =
// ((r & 3) << 2) | ((r >> 2) & 3).  With that, both access patterns are free of
// bank conflicts on the same tile:
//   row_frag : MFMA operand whose k index is the channel  (one ds_read_b128)
//   tr_frag  : MFMA operand whose k index is the row      (two ds_read_b64_tr_b16)
// Tiles are filled straight from HBM/L2 (buffer_load ... lds): a lane's 16 bytes
// land at wave_base + 16 * lane, so the swizzle is applied by choosing WHICH
// global chunk each lane fetches.  Rows past the end of the buffer descriptor
// arrive as zeros.
#pragma once
#include "common.h"

namespace beagle {
namespace tiles {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr int HD = 128;                 // head width = elements per tile row
constexpr float LOG2E = 1.44269504088896340736f;

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// Buffer descriptor over `rows` rows of 128 channels that are `stride` elements apart.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_rsrc(const bf16_t* base, int rows, int64_t stride) {
  const int64_t bytes = rows > 0 ? ((int64_t)(rows - 1) * stride + HD) * 2 : 0;
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

// Fill a tile of R rows (R * 16 chunks, 256 threads) with global rows row0 .. row0 + R - 1.
template <int R>
__device__ __forceinline__ void load_rows(bf16_t* tile, __amdgpu_buffer_rsrc_t rsrc, int64_t stride, int row0, int tid) {
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
  for (int i = 0; i < R * 16 / 256; ++i) {
    const int q = tid + 256 * i, r = q >> 4, c = (q & 15) ^ swz(r);
    const int off = (int)(((int64_t)(row0 + r) * stride + 8 * c) * 2);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(tile + (i * 4 + wave) * 512), 16, off, 0, 0, 0);
  }
}

// Per-lane element offsets of the two fragment kinds, computed once.  Tile
// bases, 32-row blocks and 16-row steps then add compile-time constants (they
// do not change swz), so that the reads use immediate offsets instead of one
// address register per fragment.
struct FragOffs {
  int row[8];      // row_frag: (lane % 32) * 128 + swizzled chunk of k step s
  int tr[4][2];    // tr_frag : channel block cb, rows {4 hf + 0..3} and {8 + 4 hf + 0..3}
};

__device__ __forceinline__ FragOffs make_frag_offs(int lane) {
  FragOffs f;
  const int ql = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int s = 0; s < 8; ++s) f.row[s] = ql * HD + (((2 * s + hf) ^ swz(ql)) << 3);
  const int gi = lane >> 4, r = lane & 15;
  const int row = 4 * (gi >> 1) + (r >> 2);
  const int sub = 4 * (r & 1);
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) {
    const int chunk = 4 * cb + 2 * (gi & 1) + ((r & 3) >> 1);
    f.tr[cb][0] = row * HD + ((chunk ^ swz(row)) << 3) + sub;
    f.tr[cb][1] = (row + 8) * HD + ((chunk ^ swz(row + 8)) << 3) + sub;
  }
  return f;
}

// whole-row fragment: row 32 * blk + lane % 32, channels 16 s + 8 hf .. + 7  (k index = channel)
__device__ __forceinline__ bf16x8_t row_frag(const bf16_t* tile, const FragOffs& f, int blk, int s) {
  return *(const bf16x8_t*)(tile + blk * 32 * HD + f.row[s]);
}

// transpose fragment: lane gets rows rowbase + {4 hf + 0..3, 8 + 4 hf + 0..3} of channel 32 cb + lane % 32
// (k index = row).  With rowbase = 32 * blk + 16 * t (a multiple of 16) this is exactly the key/query order
// of accumulator registers 8t .. 8t+7 of a 32x32 MFMA output block.
__device__ __forceinline__ bf16x8_t tr_frag(const bf16_t* tile, const FragOffs& f, int rowbase, int cb) {
  union { struct { s16x4_t x, y; } s; bf16x8_t v; } u;
  u.s.x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + rowbase * HD + f.tr[cb][0]));
  u.s.y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + rowbase * HD + f.tr[cb][1]));
  return u.v;
}

// Maximum / sum of a value over a lane and its partner lane ^ 32, in every lane.  v_permlane32_swap exchanges the
// upper half of one register with the lower half of another: fed the same value twice, every lane ends up with its
// own value in one result and its partner's in the other -- one vector instruction instead of a trip through the
// LDS crossbar (ds_bpermute), which sat on the critical path of every softmax step.
__device__ __forceinline__ float half_pair_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_pair_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ uint32_t cvt_pk(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return *(uint32_t*)&b;
}

// Workgroup id -> (row, tile position) for a staircase-shaped workload: `rows`
// independent (batch, head) rows, each with tiles of decreasing cost along the
// tile position.  Ids are dealt round-robin to the 8 XCDs, so: every XCD gets
// the same mix of tile positions (balanced), positions are visited heavy-first
// chip-wide, and all tiles of one row land on one XCD (its K/V stay in that L2).
__device__ __forceinline__ void map_block(int n, int rows, int& row, int& tpos) {
  if (rows % 8 == 0) {
    const int c = n & 7, i = n >> 3, r8 = rows >> 3;
    row = (i % r8) * 8 + c;
    tpos = i / r8;
  } else {
    row = n % rows;
    tpos = n / rows;
  }
}

// Issue-order hints for a run of N MFMAs that each consume RPM LDS reads (1 for
// a whole-row fragment, 2 for a transpose fragment): keep four fragments in
// flight ahead of the MFMA that uses them instead of read-wait-MFMA per step.
// The caller fences the run with __builtin_amdgcn_sched_barrier(0) on both sides.
template <int N, int RPM>
__device__ __forceinline__ void pipeline_reads_mfma() {
  __builtin_amdgcn_sched_group_barrier(0x100, 4 * RPM, 0);
#pragma unroll
  for (int i = 0; i < N - 4; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
}

// The same run with the first NL MFMAs each followed by one HBM -> LDS request: all waves of a workgroup pass
// the barrier together, and requests issued in one burst right behind it queue up in the CU's address unit
// (a 1 KB request takes it 16 cycles) while the waves' MFMAs wait behind them in program order.
template <int N, int RPM, int NL>
__device__ __forceinline__ void pipeline_reads_mfma_loads() {
  static_assert(NL <= N - 4, "requests ride on the MFMAs that still have reads to issue");
  __builtin_amdgcn_sched_group_barrier(0x100, 4 * RPM, 0);
#pragma unroll
  for (int i = 0; i < N - 4; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
    if (i < NL) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
}

// The same run with V vector instructions (ordinary or transcendental) of independent work slotted
// in after every MFMA, so that they issue while the matrix pipe is busy.
template <int N, int RPM, int V>
__device__ __forceinline__ void pipeline_reads_mfma_valu() {
  __builtin_amdgcn_sched_group_barrier(0x100, 4 * RPM, 0);
#pragma unroll
  for (int i = 0; i < N - 4; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
    __builtin_amdgcn_sched_group_barrier(0x402, V, 0);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x402, V, 0);
  }
}

// A wave's 32 rows x 128 channels from the accumulator layout of a transposed 32x32 MFMA block row (lane = row
// lane % 32; its registers are groups of four consecutive channels, piece 4 cb + qd = channels 32 cb + 8 qd + 4 hf ..)
// out as whole rows of a bf16 tensor.  Stored from the registers, every instruction would write 16 bytes into each of
// 32 rows; through 8 KB of LDS private to the wave instead: 8-byte pieces in, with 16-byte chunk c of row r at chunk
// c ^ (r % 16) so that the rows of an instruction spread over the banks, then whole 256-byte rows out, four rows per
// instruction.  Rows from rows_ok on are not stored.  The caller sees to it that nobody else uses the region.
__device__ __forceinline__ void store_rows_via_lds(bf16_t* region, const uint2 (&pieces)[16], int lane, bf16_t* row0,
                                                   int64_t stride, int rows_ok) {
  const int ql = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int i = 0; i < 16; ++i) *(uint2*)(region + ql * HD + ((i ^ (ql & 15)) << 3) + 4 * hf) = pieces[i];
  const int rr = lane >> 4, p = lane & 15;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = 4 * it + rr, c = p ^ (r & 15);
    const uint4 v = *(const uint4*)(region + r * HD + 8 * p);
    if (r < rows_ok) *(uint4*)(row0 + r * stride + 8 * c) = v;
  }
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt in
// bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).  Memory loads complete in
// order, so vmcnt(N) means "all but the N youngest loads have landed".
template <int N>
__device__ __forceinline__ void wait_vmem_n() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_vmem() { wait_vmem_n<0>(); }

// Workgroup barrier that orders LDS traffic only: this wave's LDS instructions have completed,
// then all waves meet.  Unlike __syncthreads() it carries no fence, so the compiler does not add
// a wait for every HBM -> LDS request that is still in flight; the caller waits for the requests
// it needs with wait_vmem_n first.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

}  // namespace tiles
}  // namespace beagle
