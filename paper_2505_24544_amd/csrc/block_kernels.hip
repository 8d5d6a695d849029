// The streaming (HBM-bound) pieces of the draft block around the cross-attention
// (section 4.1, Eq. 1): RMS normalisation of the sublayer inputs and the gate of
// the feed-forward layer, forward and backward.  Everything GEMM-shaped in the
// block runs in the GEMM kernels (the two residual adds of Eq. 1 are their
// epilogue operand); what is left touches every element once or twice, so
// these kernels are laid out for 16-byte accesses and nothing else:
//   rmsnorm_fwd   : one workgroup per row, two passes over the row (the second
//                   one hits L2), writes the normalised row and 1/rms
//   rmsnorm_bwd   : one workgroup per slice of rows; dx per row, the gain's
//                   gradient as per-workgroup column partials in LDS that a
//                   second kernel sums in a fixed order (deterministic, no
//                   atomics)
//   silu_mul_fwd / _bwd : element-wise
// Templated on the storage type (float, or bf16 bits widened on load).
#include "common.h"

namespace beagle {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of storage <-> floats
template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void ld(const float* p, float* f) {
    const f32x4 v = *(const f32x4*)p;
    f[0] = v[0]; f[1] = v[1]; f[2] = v[2]; f[3] = v[3];
  }
  static __device__ __forceinline__ void st(float* p, const float* f) {
    f32x4 v = {f[0], f[1], f[2], f[3]};
    *(f32x4*)p = v;
  }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void ld(const bf16_t* p, float* f) {
    const u32x4 w = *(const u32x4*)p;
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
  static __device__ __forceinline__ void st(bf16_t* p, const float* f) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
    *(u32x4*)p = w;
  }
};

// Sum over the 256 threads of a workgroup; every thread gets the total.
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const int wave = threadIdx.x >> 6;
  __syncthreads();                      // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// out = x / sqrt(mean(x^2) + eps) * gain, rinv[row] = 1 / sqrt(mean(x^2) + eps)
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gain,
                                                          T* __restrict__ out, float* __restrict__ rinv, int D,
                                                          float eps) {
  __shared__ float red[4];
  constexpr int N = Vec<T>::N;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * D;
  float ss = 0.f;
  for (int c = threadIdx.x * N; c < D; c += 256 * N) {
    float f[N];
    Vec<T>::ld(xr + c, f);
#pragma unroll
    for (int i = 0; i < N; ++i) ss = fmaf(f[i], f[i], ss);
  }
  const float r = 1.f / sqrtf(block_sum(ss, red) / (float)D + eps);
  if (threadIdx.x == 0) rinv[row] = r;
  for (int c = threadIdx.x * N; c < D; c += 256 * N) {
    float f[N], g[N];
    Vec<T>::ld(xr + c, f);
    Vec<T>::ld(gain + c, g);
#pragma unroll
    for (int i = 0; i < N; ++i) f[i] = f[i] * r * g[i];
    Vec<T>::st(out + row * D + c, f);
  }
}

// dx = r * (dxh - xh * mean(dxh * xh)) [+ add], dxh = dout * gain, xh = x * r;
// part[blockIdx.x][c] = sum over this workgroup's rows of dout * xh.  dx may be dout (in place: a thread
// writes only elements it has read itself, after the row's reduction).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* dout, const T* __restrict__ x,
                                                          const T* __restrict__ gain, const float* __restrict__ rinv,
                                                          const T* __restrict__ add, T* dx,
                                                          float* __restrict__ part, int rows, int D) {
  extern __shared__ float colsum[];     // [D]
  __shared__ float red[4];
  constexpr int N = Vec<T>::N;
  for (int c = threadIdx.x; c < D; c += 256) colsum[c] = 0.f;
  __syncthreads();     // from here on a thread only touches the columns it owns
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const T* dr = dout + row * D;
    const T* xr = x + row * D;
    const float r = rinv[row];
    float dot = 0.f;
    for (int c = threadIdx.x * N; c < D; c += 256 * N) {
      float a[N], b[N], g[N];
      Vec<T>::ld(dr + c, a);
      Vec<T>::ld(xr + c, b);
      Vec<T>::ld(gain + c, g);
#pragma unroll
      for (int i = 0; i < N; ++i) dot = fmaf(a[i] * g[i], b[i] * r, dot);
    }
    const float mean = block_sum(dot, red) / (float)D;
    for (int c = threadIdx.x * N; c < D; c += 256 * N) {
      float a[N], b[N], g[N], o[N];
      Vec<T>::ld(dr + c, a);
      Vec<T>::ld(xr + c, b);
      Vec<T>::ld(gain + c, g);
      if (add) Vec<T>::ld(add + row * D + c, o);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float xh = b[i] * r;
        const float v = r * (a[i] * g[i] - xh * mean);
        o[i] = add ? o[i] + v : v;
        colsum[c + i] += a[i] * xh;
      }
      Vec<T>::st(dx + row * D + c, o);
    }
  }
  for (int c = threadIdx.x * N; c < D; c += 256 * N)
#pragma unroll
    for (int i = 0; i < N; ++i) part[(int64_t)blockIdx.x * D + c + i] = colsum[c + i];
}

// out[c] = sum_p part[p][c] in a fixed order: a workgroup owns 64 columns, its four waves each sum every
// fourth partial row (eight independent loads in flight), then the four sums are added in wave order.
__global__ __launch_bounds__(256) void colsum_reduce_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                            int nparts, int D, int accumulate) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (c < D) {
    int p = wave;
    for (; p + 28 < nparts; p += 32) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = part[(int64_t)(p + 4 * i) * D + c];
#pragma unroll
      for (int i = 0; i < 8; ++i) s += v[i];
    }
    for (; p < nparts; p += 4) s += part[(int64_t)p * D + c];
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && c < D) {
    const float t = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
    out[c] = accumulate ? out[c] + t : t;      // a gain shared by two normalised inputs collects both
  }
}

__device__ __forceinline__ float sigmoidf(float u) { return 1.f / (1.f + expf(-u)); }

// m = silu(u) * w
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_fwd_kernel(const T* __restrict__ u, const T* __restrict__ w,
                                                           T* __restrict__ m, int64_t n) {
  constexpr int N = Vec<T>::N;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * N; i < n; i += (int64_t)gridDim.x * 256 * N) {
    float a[N], b[N];
    Vec<T>::ld(u + i, a);
    Vec<T>::ld(w + i, b);
#pragma unroll
    for (int k = 0; k < N; ++k) a[k] = a[k] * sigmoidf(a[k]) * b[k];
    Vec<T>::st(m + i, a);
  }
}

// du = dm * w * sig(u) * (1 + u * (1 - sig(u))), dw = dm * u * sig(u); du may be dm (in place)
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_bwd_kernel(const T* dm, const T* __restrict__ u,
                                                           const T* __restrict__ w, T* du, T* __restrict__ dw,
                                                           int64_t n) {
  constexpr int N = Vec<T>::N;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * N; i < n; i += (int64_t)gridDim.x * 256 * N) {
    float g[N], a[N], b[N], x[N], y[N];
    Vec<T>::ld(dm + i, g);
    Vec<T>::ld(u + i, a);
    Vec<T>::ld(w + i, b);
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const float sg = sigmoidf(a[k]);
      x[k] = g[k] * b[k] * sg * (1.f + a[k] * (1.f - sg));
      y[k] = g[k] * a[k] * sg;
    }
    Vec<T>::st(du + i, x);
    Vec<T>::st(dw + i, y);
  }
}

// IEEE half -> storage type, eight elements per thread and step (the offline-generated target states arrive in
// half precision: section 5.1, experimental set-up)
template <typename T>
__global__ __launch_bounds__(256) void cvt_f16_kernel(const _Float16* __restrict__ in, T* __restrict__ out, int64_t n) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8; i < n; i += (int64_t)gridDim.x * 256 * 8) {
    const h8 v = *(const h8*)(in + i);
    float f[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) f[k] = (float)v[k];
    if (sizeof(T) == 2) {
      Vec<bf16_t>::st((bf16_t*)out + i, f);
    } else {
      Vec<float>::st((float*)out + i, f);
      Vec<float>::st((float*)out + i + 4, f + 4);
    }
  }
}

template <typename T>
void rmsnorm_fwd_t(const void* x, const void* gain, void* out, float* rinv, int64_t rows, int D, float eps, hipStream_t s) {
  hipLaunchKernelGGL(rmsnorm_fwd_kernel<T>, dim3((unsigned)rows), dim3(256), 0, s, (const T*)x, (const T*)gain, (T*)out,
                     rinv, D, eps);
}
template <typename T>
void rmsnorm_bwd_t(const void* dout, const void* x, const void* gain, const float* rinv, const void* add, void* dx,
                   float* dgain, float* part, int nparts, int64_t rows, int D, bool accumulate, hipStream_t s) {
  hipLaunchKernelGGL(rmsnorm_bwd_kernel<T>, dim3(nparts), dim3(256), (size_t)D * sizeof(float), s, (const T*)dout,
                     (const T*)x, (const T*)gain, rinv, (const T*)add, (T*)dx, part, (int)rows, D);
  hipLaunchKernelGGL(colsum_reduce_kernel, dim3((D + 63) / 64), dim3(256), 0, s, part, dgain, nparts, D, accumulate ? 1 : 0);
}

int elementwise_grid(int64_t n, int per_thread) {
  const int64_t blocks = (n / per_thread + 255) / 256;
  return (int)(blocks < 1 ? 1 : (blocks > 16384 ? 16384 : blocks));
}

}  // namespace

int rmsnorm_bwd_parts(int64_t rows) { return (int)(rows < RMS_BWD_MAX_PARTS ? rows : RMS_BWD_MAX_PARTS); }

void launch_rmsnorm_fwd(bool bf16, const void* x, const void* gain, void* out, float* rinv, int64_t rows, int D,
                        float eps, hipStream_t s, const char* name) {
  ProfScope ps(name, s);
  if (bf16) rmsnorm_fwd_t<bf16_t>(x, gain, out, rinv, rows, D, eps, s);
  else rmsnorm_fwd_t<float>(x, gain, out, rinv, rows, D, eps, s);
}

void launch_rmsnorm_bwd(bool bf16, const void* dout, const void* x, const void* gain, const float* rinv,
                        const void* add, void* dx, float* dgain, float* part, int64_t rows, int D, hipStream_t s,
                        const char* name, bool accumulate) {
  ProfScope ps(name, s);
  const int nparts = rmsnorm_bwd_parts(rows);
  if (bf16) rmsnorm_bwd_t<bf16_t>(dout, x, gain, rinv, add, dx, dgain, part, nparts, rows, D, accumulate, s);
  else rmsnorm_bwd_t<float>(dout, x, gain, rinv, add, dx, dgain, part, nparts, rows, D, accumulate, s);
}

void launch_cvt_f16(bool bf16, const void* in, void* out, int64_t n, hipStream_t s) {
  ProfScope ps("states_f16", s);
  if (bf16) hipLaunchKernelGGL(cvt_f16_kernel<bf16_t>, dim3(elementwise_grid(n, 8)), dim3(256), 0, s, (const _Float16*)in,
                               (bf16_t*)out, n);
  else hipLaunchKernelGGL(cvt_f16_kernel<float>, dim3(elementwise_grid(n, 8)), dim3(256), 0, s, (const _Float16*)in,
                          (float*)out, n);
}

void launch_silu_mul_fwd(bool bf16, const void* u, const void* w, void* m, int64_t n, hipStream_t s) {
  ProfScope ps("mlp_gate", s);
  if (bf16) hipLaunchKernelGGL(silu_mul_fwd_kernel<bf16_t>, dim3(elementwise_grid(n, 8)), dim3(256), 0, s,
                               (const bf16_t*)u, (const bf16_t*)w, (bf16_t*)m, n);
  else hipLaunchKernelGGL(silu_mul_fwd_kernel<float>, dim3(elementwise_grid(n, 4)), dim3(256), 0, s, (const float*)u,
                          (const float*)w, (float*)m, n);
}

void launch_silu_mul_bwd(bool bf16, const void* dm, const void* u, const void* w, void* du, void* dw, int64_t n,
                         hipStream_t s) {
  ProfScope ps("bwd_mlp_gate", s);
  if (bf16) hipLaunchKernelGGL(silu_mul_bwd_kernel<bf16_t>, dim3(elementwise_grid(n, 8)), dim3(256), 0, s,
                               (const bf16_t*)dm, (const bf16_t*)u, (const bf16_t*)w, (bf16_t*)du, (bf16_t*)dw, n);
  else hipLaunchKernelGGL(silu_mul_bwd_kernel<float>, dim3(elementwise_grid(n, 4)), dim3(256), 0, s, (const float*)dm,
                          (const float*)u, (const float*)w, (float*)du, (float*)dw, n);
}

}  // namespace beagle
