// Plain streaming kernels of known size: what this memory system gives to the simplest code,
// measured beside the path's kernels so that their rates can be placed against it (and not
// only against the published 8 TB/s).  Not part of the method and not part of libwcc: this file
// is the whole of libwcc_probe.so, a measurement aid that bench.py loads.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>

#include "wcc_probe.h"

namespace {

typedef float vf4 __attribute__((ext_vector_type(4)));
constexpr int kProbeBlocks = 8192;  // default: 32 workgroups a CU, grid-stride

template <bool NT>
__device__ __forceinline__ vf4 probe_load(const vf4 *p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT>
__device__ __forceinline__ void probe_store(vf4 *p, vf4 v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Reads n 16-byte words; the sum is stored only if it equals a value it cannot take, so the
// loads stay and nothing is written.
template <bool NT>
__global__ __launch_bounds__(256) void probe_read_kernel(const vf4 *__restrict__ src, size_t n,
                                                         vf4 *__restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  vf4 acc = {0.f, 0.f, 0.f, 0.f};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    acc += probe_load<NT>(src + i);
  if (acc.x == 1.2345e38f && acc.y == -1.2345e38f) sink[0] = acc;
}

// dst[i] = (1, 2, 3, 4)
template <bool NT>
__global__ __launch_bounds__(256) void probe_write_kernel(vf4 *__restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const vf4 v = {1.f, 2.f, 3.f, 4.f};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    probe_store<NT>(dst + i, v);
}

// The same fill with eight stores a thread: a workgroup writes 32 KiB in a row, every store
// instruction of it 4 KiB (what a kernel does whose waves own several rows of a tile; the rate
// drops with the stores per thread although the bytes and their order in memory are the same).
template <bool NT>
__global__ __launch_bounds__(256) void probe_write8_kernel(vf4 *__restrict__ dst, size_t n) {
  const size_t first = (size_t)blockIdx.x * (256 * 8) + threadIdx.x;
  const vf4 v = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const size_t i = first + (size_t)r * 256;
    if (i < n) probe_store<NT>(dst + i, v);
  }
}

template <bool NT>
__global__ __launch_bounds__(256) void probe_copy_kernel(const vf4 *__restrict__ src,
                                                         vf4 *__restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    probe_store<NT>(dst + i, probe_load<NT>(src + i));
}

}  // namespace

extern "C" int wcc_probe_stream(int kind, const void *src, void *dst, size_t bytes, int nontemporal,
                                int blocks, void *stream) {
  if (kind < WCC_PROBE_READ || kind > WCC_PROBE_WRITE8) return WCC_PROBE_ERR_KIND;
  const bool writes_only = kind == WCC_PROBE_WRITE || kind == WCC_PROBE_WRITE8;
  if (!dst || (!writes_only && !src)) return WCC_PROBE_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0 || blocks < 0 || blocks > (1 << 24)) return WCC_PROBE_ERR_SIZE;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return WCC_PROBE_ERR_SIZE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool nt = nontemporal != 0;
  const size_t n = bytes / 16;
  const vf4 *in = static_cast<const vf4 *>(src);
  vf4 *out = static_cast<vf4 *>(dst);
  const dim3 grid((unsigned)std::min<size_t>(blocks > 0 ? blocks : kProbeBlocks, (n + 255) / 256)), block(256);
  switch (kind) {
    case WCC_PROBE_READ:
      if (nt) hipLaunchKernelGGL(probe_read_kernel<true>, grid, block, 0, s, in, n, out);
      else hipLaunchKernelGGL(probe_read_kernel<false>, grid, block, 0, s, in, n, out);
      break;
    case WCC_PROBE_WRITE:
      if (nt) hipLaunchKernelGGL(probe_write_kernel<true>, grid, block, 0, s, out, n);
      else hipLaunchKernelGGL(probe_write_kernel<false>, grid, block, 0, s, out, n);
      break;
    case WCC_PROBE_COPY:
      if (nt) hipLaunchKernelGGL(probe_copy_kernel<true>, grid, block, 0, s, in, out, n);
      else hipLaunchKernelGGL(probe_copy_kernel<false>, grid, block, 0, s, in, out, n);
      break;
    default: {
      if ((n + 2047) / 2048 > 0x7FFFFFFFull) return WCC_PROBE_ERR_SIZE;
      const dim3 g8((unsigned)((n + 2047) / 2048));
      if (nt) hipLaunchKernelGGL(probe_write8_kernel<true>, g8, block, 0, s, out, n);
      else hipLaunchKernelGGL(probe_write8_kernel<false>, g8, block, 0, s, out, n);
      break;
    }
  }
  return hipGetLastError() == hipSuccess ? WCC_PROBE_OK : WCC_PROBE_ERR_HIP;
}
