// Rotary position embedding of projected queries / keys, in place (optional;
// section 4.1 leaves positional embeddings out of its equations, the LLaMA /
// Vicuna targets rotate Q and K).  Rotate-half convention: channel c < d/2 of a
// head is paired with channel c + d/2, angle = position * base^(-2c/d); the
// inverse rotation (the transpose) is what the backward pass applies to dQ, dK.
//
// Streaming kernel (bound: HBM): one workgroup per row (all heads of one
// position), a thread owns two adjacent channel pairs of every eighth head, so
// the angle's sine and cosine -- evaluated in double, which keeps the fp32 path
// within 1e-5 at positions in the thousands -- are computed twice per thread
// per row and reused for all heads.  Up to three tensors share one launch.
#include "common.h"

namespace beagle {
namespace {

template <typename T> struct Pair2;
template <> struct Pair2<float> {
  static __device__ __forceinline__ void ld(const float* p, float& a, float& b) { const float2 v = *(const float2*)p; a = v.x; b = v.y; }
  static __device__ __forceinline__ void st(float* p, float a, float b) { *(float2*)p = make_float2(a, b); }
};
template <> struct Pair2<bf16_t> {
  static __device__ __forceinline__ void ld(const bf16_t* p, float& a, float& b) {
    const uint32_t w = *(const uint32_t*)p;
    a = __uint_as_float(w << 16); b = __uint_as_float(w & 0xffff0000u);
  }
  static __device__ __forceinline__ void st(bf16_t* p, float a, float b) { *(uint32_t*)p = pack_bf16x2(a, b); }
};

template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(RopeArgs r) {
  int seg = 0;
  int64_t row = blockIdx.x;
  while (seg + 1 < r.n && row >= r.rows[seg]) { row -= r.rows[seg]; ++seg; }
  const int d = r.d, half = d >> 1, lanes = half >> 1;          // lanes per head: two channel pairs each
  const int c = 2 * (threadIdx.x % 32), hg = threadIdx.x / 32;   // first channel of this thread, head group
  if (c >= half) return;
  (void)lanes;
  int idx = (int)(row % r.period[seg]);
  if (r.cu[seg]) {                               // packed batch: the entry whose rows include this one
    const int32_t* cu = r.cu[seg];
    int lo = 0, hi = r.nb;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (cu[mid] <= row) lo = mid; else hi = mid;
    }
    idx = (int)(row - cu[lo]);
  }
  const int pos = r.pos[seg] ? r.pos[seg][idx] : r.pos0[seg] + idx;
  double s0, c0, s1, c1;
  const double l2b = log2((double)r.base);
  sincos((double)pos * exp2(-2.0 * c / d * l2b), &s0, &c0);
  sincos((double)pos * exp2(-2.0 * (c + 1) / d * l2b), &s1, &c1);
  if (r.inverse) { s0 = -s0; s1 = -s1; }
  const float fs0 = (float)s0, fc0 = (float)c0, fs1 = (float)s1, fc1 = (float)c1;
  T* x = (T*)r.x[seg] + row * (int64_t)r.heads[seg] * d;
  for (int h = hg; h < r.heads[seg]; h += 8) {
    T* p = x + h * d + c;
    float a0, a1, b0, b1;
    Pair2<T>::ld(p, a0, a1);
    Pair2<T>::ld(p + half, b0, b1);
    Pair2<T>::st(p, a0 * fc0 - b0 * fs0, a1 * fc1 - b1 * fs1);
    Pair2<T>::st(p + half, b0 * fc0 + a0 * fs0, b1 * fc1 + a1 * fs1);
  }
}

}  // namespace

void launch_rope(bool bf16, const RopeArgs& r, hipStream_t s, const char* name) {
  int64_t total = 0;
  for (int i = 0; i < r.n; ++i) total += r.rows[i];
  if (total == 0) return;
  ProfScope ps(name, s);
  if (bf16) hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3((unsigned)total), dim3(256), 0, s, r);
  else hipLaunchKernelGGL(rope_kernel<float>, dim3((unsigned)total), dim3(256), 0, s, r);
}

}  // namespace beagle
