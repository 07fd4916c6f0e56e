// Shrinkage operator T applied with one index list to every channel (Eq. T, Alg. 1:
// X_wt[I]), the layer-wide clipping parameter alpha = max |kept coefficient|, and the signed
// uniform quantiser of Eq. (quantweights) with b = 8.
#include "wcc_internal.h"

namespace wcc {
namespace {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_down(v, off, 64));
  return v;
}

// alpha[0] = alpha_in if positive, else 0 (then raised by the gather's max reduction)
__global__ void alpha_init_kernel(float *alpha, float alpha_in) {
  if (threadIdx.x == 0) alpha[0] = alpha_in > 0.f ? alpha_in : 0.f;
}

// xc[b, c, j] = coef[b, c, idx[b, j]].  grid = (ceil(k / 1024), C, B), block = 256, four
// consecutive j per thread.  VEC: k is a multiple of 4 (16-byte idx loads and xc stores).
template <bool VEC>
__global__ __launch_bounds__(256) void gather_kernel(const float *__restrict__ coef,
                                                     const int32_t *__restrict__ idx, int C,
                                                     int64_t N, int64_t k, float *__restrict__ xc,
                                                     float *alpha_max) {
  __shared__ float wmax[4];
  const int c = blockIdx.y, b = blockIdx.z;
  const int64_t j0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const float *plane = coef + ((size_t)b * C + c) * N;
  const int32_t *ix = idx + (size_t)b * k;
  float *out = xc + ((size_t)b * C + c) * k;
  float m = 0.f;
  if (j0 < k) {
    if constexpr (VEC) {
      int4 q = *reinterpret_cast<const int4 *>(ix + j0);
      const int hi = (int)N - 1;  // an out-of-range index never leaves the plane
      q.x = min(max(q.x, 0), hi); q.y = min(max(q.y, 0), hi);
      q.z = min(max(q.z, 0), hi); q.w = min(max(q.w, 0), hi);
      float4 v;
      v.x = plane[q.x]; v.y = plane[q.y]; v.z = plane[q.z]; v.w = plane[q.w];
      *reinterpret_cast<float4 *>(out + j0) = v;
      m = fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));
    } else {
      for (int e = 0; e < 4 && j0 + e < k; ++e) {
        const float v = plane[min(max(ix[j0 + e], 0), (int)N - 1)];
        out[j0 + e] = v;
        m = fmaxf(m, fabsf(v));
      }
    }
  }
  if (alpha_max == nullptr) return;
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    // non-negative floats order like their bit patterns: an integer max is exact and
    // independent of arrival order
    if (m > 0.f) atomicMax(reinterpret_cast<unsigned int *>(alpha_max), __float_as_uint(m));
  }
}

// The scale-clip-round of Eq. (quantweights), signed, b = 8, operation by operation in fp32.
__device__ __forceinline__ int quant_code(float v, float alpha) {
  if (!(alpha > 0.f)) return 0;
  float u = __fdiv_rn(v, alpha);          // scale
  u = fminf(fmaxf(u, -1.f), 1.f);         // clip
  return (int)rintf(__fmul_rn(127.f, u)); // round half to even
}

// codes[i] = q(xc32[i]); 16 values per thread when n is a multiple of 16
__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ xc32, int64_t n,
                                                       const float *__restrict__ alpha,
                                                       int8_t *__restrict__ codes) {
  const float a = alpha[0];
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (i0 >= n) return;
  if (i0 + 16 <= n && (n & 15) == 0) {
    uint32_t packed[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = *reinterpret_cast<const float4 *>(xc32 + i0 + 4 * g);
      const uint32_t c0 = (uint32_t)quant_code(v.x, a) & 0xFFu, c1 = (uint32_t)quant_code(v.y, a) & 0xFFu;
      const uint32_t c2 = (uint32_t)quant_code(v.z, a) & 0xFFu, c3 = (uint32_t)quant_code(v.w, a) & 0xFFu;
      packed[g] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
    }
    *reinterpret_cast<uint4 *>(codes + i0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
  } else {
    for (int e = 0; e < 16 && i0 + e < n; ++e) codes[i0 + e] = (int8_t)quant_code(xc32[i0 + e], a);
  }
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float *__restrict__ src,
                                                       float *__restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

}  // namespace

hipError_t launch_alpha_init(float *alpha, float alpha_in, hipStream_t s) {
  hipLaunchKernelGGL(alpha_init_kernel, dim3(1), dim3(64), 0, s, alpha, alpha_in);
  return hipGetLastError();
}

hipError_t launch_gather(const float *coef, const int32_t *idx, int B, int C, int64_t N, int64_t k,
                         float *xc, float *alpha_max, hipStream_t s) {
  dim3 grid((unsigned)((k + 1023) / 1024), C, B);
  if (k % 4 == 0)
    hipLaunchKernelGGL(gather_kernel<true>, grid, dim3(256), 0, s, coef, idx, C, N, k, xc, alpha_max);
  else
    hipLaunchKernelGGL(gather_kernel<false>, grid, dim3(256), 0, s, coef, idx, C, N, k, xc, alpha_max);
  return hipGetLastError();
}

hipError_t launch_quantize(const float *xc32, int64_t n, const float *alpha, int8_t *codes,
                           hipStream_t s) {
  hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)((n + 4095) / 4096)), dim3(256), 0, s, xc32, n,
                     alpha, codes);
  return hipGetLastError();
}

hipError_t launch_copy_f32(const float *src, float *dst, int64_t n, hipStream_t s) {
  hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dst, n);
  return hipGetLastError();
}

}  // namespace wcc
