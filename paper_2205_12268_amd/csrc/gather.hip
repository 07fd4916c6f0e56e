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

// every slot = alpha_in if positive, else 0 (then raised by the gather's max reduction)
__global__ void alpha_init_kernel(float *slots, float alpha_in) {
  if (threadIdx.x < kAlphaSlots) slots[threadIdx.x] = alpha_in > 0.f ? alpha_in : 0.f;
}

constexpr int kGatherIters = 4;  // a workgroup covers 4 x 1024 consecutive j

// xc[b, c, j] = coef[b, c, idx[b, j]].  grid = (ceil(k / 4096), C, B), block = 256, four
// consecutive j per thread and iteration.  VEC: k is a multiple of 4 (16-byte idx loads and
// xc stores).
template <bool VEC>
__global__ __launch_bounds__(256) void gather_kernel(const float *__restrict__ coef,
                                                     const int32_t *__restrict__ idx, int C,
                                                     int64_t N, int64_t k, float *__restrict__ xc,
                                                     float *alpha_slots) {
  __shared__ float wmax[4];
  const int c = blockIdx.y, b = blockIdx.z;
  const float *plane = coef + ((size_t)b * C + c) * N;
  const int32_t *ix = idx + (size_t)b * k;
  float *out = xc + ((size_t)b * C + c) * k;
  float m = 0.f;
  const int hi = (int)N - 1;  // an out-of-range index never leaves the plane
  if constexpr (VEC) {
    // all index loads first, then all gathers, then the stores: 16 independent loads in flight
    int4 q[kGatherIters];
    int64_t j0[kGatherIters];
#pragma unroll
    for (int it = 0; it < kGatherIters; ++it) {
      j0[it] = (((int64_t)blockIdx.x * kGatherIters + it) * 256 + threadIdx.x) * 4;
      q[it] = make_int4(0, 0, 0, 0);
      if (j0[it] < k) q[it] = *reinterpret_cast<const int4 *>(ix + j0[it]);
    }
    float4 v[kGatherIters];
#pragma unroll
    for (int it = 0; it < kGatherIters; ++it) {
      v[it].x = plane[min(max(q[it].x, 0), hi)];
      v[it].y = plane[min(max(q[it].y, 0), hi)];
      v[it].z = plane[min(max(q[it].z, 0), hi)];
      v[it].w = plane[min(max(q[it].w, 0), hi)];
    }
#pragma unroll
    for (int it = 0; it < kGatherIters; ++it) {
      if (j0[it] < k) {
        *reinterpret_cast<float4 *>(out + j0[it]) = v[it];
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v[it].x), fabsf(v[it].y)), fmaxf(fabsf(v[it].z), fabsf(v[it].w))));
      }
    }
  } else {
    for (int it = 0; it < kGatherIters; ++it) {
      const int64_t j0 = (((int64_t)blockIdx.x * kGatherIters + it) * 256 + threadIdx.x) * 4;
      for (int e = 0; e < 4 && j0 + e < k; ++e) {
        const float v = plane[min(max(ix[j0 + e], 0), hi)];
        out[j0 + e] = v;
        m = fmaxf(m, fabsf(v));
      }
    }
  }
  if (alpha_slots == nullptr) return;
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    // Non-negative floats order like their bit patterns: an integer max is exact and
    // independent of arrival order.  Atomics on one address serialise at the memory side, so
    // the workgroups spread over kAlphaSlots addresses; the consumer takes the max of the
    // slots.  A slot only grows: a workgroup at or below the value it observes skips.
    unsigned int *a = reinterpret_cast<unsigned int *>(alpha_slots) +
                      ((blockIdx.x + 3u * blockIdx.y + 11u * blockIdx.z) & (kAlphaSlots - 1));
    const unsigned int mine = __float_as_uint(m);
    if (mine > __hip_atomic_load(a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(a, mine);
  }
}

// codes[i] = q(xc32[i]); 16 values per thread when n is a multiple of 16
__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ xc32, int64_t n,
                                                       const float *__restrict__ alpha_slots,
                                                       float *__restrict__ alpha_out,
                                                       int8_t *__restrict__ codes) {
  const float alpha = alpha_max(alpha_slots, kAlphaSlots);
  if (blockIdx.x == 0 && threadIdx.x == 0) alpha_out[0] = alpha;
  const Quant a(alpha);
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (i0 >= n) return;
  if (i0 + 16 <= n && (n & 15) == 0) {
    uint32_t packed[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = *reinterpret_cast<const float4 *>(xc32 + i0 + 4 * g);
      const uint32_t c0 = (uint32_t)a.code(v.x) & 0xFFu, c1 = (uint32_t)a.code(v.y) & 0xFFu;
      const uint32_t c2 = (uint32_t)a.code(v.z) & 0xFFu, c3 = (uint32_t)a.code(v.w) & 0xFFu;
      packed[g] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
    }
    *reinterpret_cast<uint4 *>(codes + i0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
  } else {
    for (int e = 0; e < 16 && i0 + e < n; ++e) codes[i0 + e] = (int8_t)a.code(xc32[i0 + e]);
  }
}

// two signed 4-bit codes a byte (low nibble first) -> int8 codes
__global__ __launch_bounds__(256) void unpack_i4_kernel(const uint8_t *__restrict__ packed,
                                                        int8_t *__restrict__ out, int64_t n_bytes) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_bytes) return;
  const uint32_t v = packed[i];
  const int lo = (int)(v << 28) >> 28, hi = (int)(v << 24) >> 28;  // sign-extend the nibbles
  out[2 * i] = (int8_t)lo;
  out[2 * i + 1] = (int8_t)hi;
}

}  // namespace

hipError_t launch_unpack_i4(const uint8_t *packed, int8_t *out, int64_t n, hipStream_t s) {
  const int64_t nb = n / 2;
  hipLaunchKernelGGL(unpack_i4_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, s, packed, out, nb);
  return hipGetLastError();
}

hipError_t launch_alpha_init(float *alpha_slots, float alpha_in, hipStream_t s) {
  hipLaunchKernelGGL(alpha_init_kernel, dim3(1), dim3(64), 0, s, alpha_slots, alpha_in);
  return hipGetLastError();
}

hipError_t launch_gather(const float *coef, const int32_t *idx, int B, int C, int64_t N, int64_t k,
                         float *xc, float *alpha_slots, hipStream_t s) {
  dim3 grid((unsigned)((k + 1024 * kGatherIters - 1) / (1024 * kGatherIters)), C, B);
  if (k % 4 == 0)
    hipLaunchKernelGGL(gather_kernel<true>, grid, dim3(256), 0, s, coef, idx, C, N, k, xc, alpha_slots);
  else
    hipLaunchKernelGGL(gather_kernel<false>, grid, dim3(256), 0, s, coef, idx, C, N, k, xc, alpha_slots);
  return hipGetLastError();
}

hipError_t launch_quantize(const float *xc32, int64_t n, const float *alpha_slots, float *alpha_out,
                           int8_t *codes, hipStream_t s) {
  hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)((n + 4095) / 4096)), dim3(256), 0, s, xc32, n,
                     alpha_slots, alpha_out, codes);
  return hipGetLastError();
}


}  // namespace wcc
