// The 1x1 convolution on the compressed signal (Eq. WCC: K_1x1 applied between T and T^T;
// "y_i = sum_j k_ij x_j" with x_j the length-k compressed channel vectors): per sample a
// [C_out x C_in] . [C_in x k] contraction, k contiguous in memory on both sides.
//
// Matrix-core kernels (int8 activation codes):
//   bf16 weights: v_mfma_f32_32x32x16_bf16.  The int8 codes (|n| <= 127) are exact in bf16
//                 and every product is exact in fp32; only the fp32 accumulation rounds.
//   int8 weights: v_mfma_i32_32x32x32_i8, exact int32 accumulation.
// A workgroup (4 waves) computes a 128 x 128 tile; wave w owns rows 32w..32w+31 and all 128
// columns.  The activation tile arrives k-contiguous-along-n from HBM; each thread takes a
// 4(n) x 8(c) patch in registers, transposes it, and stores it to LDS with the n rows permuted
// (row (n%4)*32 + n/4) so that MFMA column c of column block i is n = 4c + i: after the four
// column blocks a lane holds four adjacent n of one output row and stores them as 16 bytes.
// Everything else (fp32 weights, unquantised activations, odd shapes) takes a plain fp32 FMA
// tile kernel on the weights widened to fp32.
#include "wcc_internal.h"

namespace wcc {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int intx4;
typedef __attribute__((__vector_size__(16 * sizeof(int)))) int intx16;

constexpr int BM = 128, BN = 128, BK = 64;

// ---- bf16 x (int8 codes as bf16) -> fp32 ----------------------------------------------------
constexpr int LDB = BK + 8;  // bf16 elements per LDS row (144 bytes: 16-byte aligned, 36 banks)

__device__ __forceinline__ uint32_t code_to_bf16(uint32_t dw, int byte) {
  const int v = (int)(dw << (24 - 8 * byte)) >> 24;  // sign-extended byte
  return __float_as_uint((float)v) >> 16;           // |v| <= 128: exact in bf16
}

// The layer's alpha: one float, or the max of the gather's slots.  The first workgroup also
// publishes it to alpha_out (nullable).  Called by every thread of the workgroup.
__device__ __forceinline__ float load_alpha(const float *__restrict__ alpha, bool slots,
                                            float *alpha_out) {
  const float a = slots ? alpha_from_slots(alpha) : alpha[0];
  if (alpha_out && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
    alpha_out[0] = a;
  return a;
}

// A thread's 8 (channels) x 4 (positions) patch of the activation tile as packed int8 codes:
// dw[r] holds positions n..n+3 of channel c0 + r.  F32: the source holds unquantised kept
// coefficients, quantised here with the layer's alpha.
template <bool F32>
__device__ __forceinline__ void load_patch(const void *__restrict__ xb, int K, int64_t k, int c0,
                                           int64_t n, float alpha, uint32_t (&dw)[8]) {
  if constexpr (F32) {
    const float *xf = static_cast<const float *>(xb);
    float4 v[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      v[r] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (c0 + r < K && n < k) v[r] = *reinterpret_cast<const float4 *>(xf + (size_t)(c0 + r) * k + n);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      dw[r] = ((uint32_t)quant_code(v[r].x, alpha) & 0xFFu) |
              (((uint32_t)quant_code(v[r].y, alpha) & 0xFFu) << 8) |
              (((uint32_t)quant_code(v[r].z, alpha) & 0xFFu) << 16) |
              (((uint32_t)quant_code(v[r].w, alpha) & 0xFFu) << 24);
    }
  } else {
    const int8_t *xq = static_cast<const int8_t *>(xb);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      dw[r] = 0;
      if (c0 + r < K && n < k) dw[r] = *reinterpret_cast<const uint32_t *>(xq + (size_t)(c0 + r) * k + n);
    }
  }
}

// grid = (ceil(k/128), ceil(M/128), B); needs K % 8 == 0 and k % 4 == 0
template <bool F32>
__global__ __launch_bounds__(256) void pointwise_bf16_kernel(const uint16_t *__restrict__ w,
                                                             const void *__restrict__ xq,
                                                             const float *__restrict__ alpha,
                                                             bool slots, float *alpha_out,
                                                             float *__restrict__ yc, int M, int K,
                                                             int64_t k) {
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDB];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDB];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const int b = blockIdx.z, m0 = blockIdx.y * BM;
  const int64_t n0 = (int64_t)blockIdx.x * BN;
  const void *xb = static_cast<const char *>(xq) + (size_t)b * K * k * (F32 ? 4 : 1);
  const float al = load_alpha(alpha, slots, alpha_out);

  floatx16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int a_row = t >> 1, a_half = t & 1;       // A loader: row, which 32 of the 64 k
  const int g = t & 31, kq = t >> 5;              // B loader: n group (4 n), k octet
  for (int k0 = 0; k0 < K; k0 += BK) {
    // weights tile: As[row][kk] = w[m0 + row][k0 + kk], zero outside
    {
      const int m = m0 + a_row;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int kk = a_half * 32 + q * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (m < M && k0 + kk < K) v = *reinterpret_cast<const uint4 *>(w + (size_t)m * K + k0 + kk);
        *reinterpret_cast<uint4 *>(&As[a_row * LDB + kk]) = v;
      }
    }
    // activation tile: 8 channels x 4 positions per thread, transposed into Bs
    {
      uint32_t dw[8];
      load_patch<F32>(xb, K, k, k0 + kq * 8, n0 + 4 * g, al, dw);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 v;
        v.x = code_to_bf16(dw[0], i) | (code_to_bf16(dw[1], i) << 16);
        v.y = code_to_bf16(dw[2], i) | (code_to_bf16(dw[3], i) << 16);
        v.z = code_to_bf16(dw[4], i) | (code_to_bf16(dw[5], i) << 16);
        v.w = code_to_bf16(dw[6], i) | (code_to_bf16(dw[7], i) << 16);
        *reinterpret_cast<uint4 *>(&Bs[(i * 32 + g) * LDB + kq * 8]) = v;
      }
    }
    __syncthreads();
    const int fr = lane & 31, fk = (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const bf16x8 a = __builtin_bit_cast(
          bf16x8, *reinterpret_cast<const uint4 *>(&As[(wv * 32 + fr) * LDB + ks * 16 + fk]));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bf16x8 bb = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4 *>(&Bs[(i * 32 + fr) * LDB + ks * 16 + fk]));
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc[i], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  // epilogue: acc[i][r] is row (r/4)*8 + (lane/32)*4 + r%4, column 4*(lane%32) + i
  const float sx = al / 127.f;
  const int64_t n = n0 + 4 * (lane & 31);
  if (n >= k) return;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = m0 + wv * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
    if (m < M) {
      const float4 v = make_float4(acc[0][r] * sx, acc[1][r] * sx, acc[2][r] * sx, acc[3][r] * sx);
      *reinterpret_cast<float4 *>(yc + ((size_t)b * M + m) * k + n) = v;
    }
  }
}

// ---- int8 x int8 -> int32 ------------------------------------------------------------------------
constexpr int LDI = BK + 16;  // bytes per LDS row (80 bytes: 16-byte aligned, 20 banks)

// byte `i` of four dwords -> one dword
__device__ __forceinline__ uint32_t gather_byte(uint32_t d0, uint32_t d1, uint32_t d2, uint32_t d3, int i) {
  const uint32_t sel = (uint32_t)i | ((uint32_t)(4 + i) << 8);
  const uint32_t lo = __builtin_amdgcn_perm(d1, d0, sel);  // [d0.b_i, d1.b_i, -, -]
  const uint32_t hi = __builtin_amdgcn_perm(d3, d2, sel);
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// grid = (ceil(k/128), ceil(M/128), B); needs K % 16 == 0 and k % 4 == 0
template <bool F32>
__global__ __launch_bounds__(256) void pointwise_i8_kernel(const int8_t *__restrict__ w,
                                                           const float *__restrict__ w_scale,
                                                           const void *__restrict__ xq,
                                                           const float *__restrict__ alpha,
                                                           bool slots, float *alpha_out,
                                                           float *__restrict__ yc, int M, int K,
                                                           int64_t k) {
  __shared__ __attribute__((aligned(16))) int8_t As[BM * LDI];
  __shared__ __attribute__((aligned(16))) int8_t Bs[BN * LDI];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const int b = blockIdx.z, m0 = blockIdx.y * BM;
  const int64_t n0 = (int64_t)blockIdx.x * BN;
  const void *xb = static_cast<const char *>(xq) + (size_t)b * K * k * (F32 ? 4 : 1);
  const float al = load_alpha(alpha, slots, alpha_out);

  intx16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0;

  const int a_row = t >> 1, a_half = t & 1;
  const int g = t & 31, kq = t >> 5;
  for (int k0 = 0; k0 < K; k0 += BK) {
    {
      const int m = m0 + a_row;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int kk = a_half * 32 + q * 16;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (m < M && k0 + kk < K) v = *reinterpret_cast<const uint4 *>(w + (size_t)m * K + k0 + kk);
        *reinterpret_cast<uint4 *>(&As[a_row * LDI + kk]) = v;
      }
    }
    {
      uint32_t dw[8];
      load_patch<F32>(xb, K, k, k0 + kq * 8, n0 + 4 * g, al, dw);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint2 v;
        v.x = gather_byte(dw[0], dw[1], dw[2], dw[3], i);
        v.y = gather_byte(dw[4], dw[5], dw[6], dw[7], i);
        *reinterpret_cast<uint2 *>(&Bs[(i * 32 + g) * LDI + kq * 8]) = v;
      }
    }
    __syncthreads();
    const int fr = lane & 31, fk = (lane >> 5) * 16;
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      const intx4 a = __builtin_bit_cast(
          intx4, *reinterpret_cast<const uint4 *>(&As[(wv * 32 + fr) * LDI + ks * 32 + fk]));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const intx4 bb = __builtin_bit_cast(
            intx4, *reinterpret_cast<const uint4 *>(&Bs[(i * 32 + fr) * LDI + ks * 32 + fk]));
        acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bb, acc[i], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  const float sx = al / 127.f;
  const int64_t n = n0 + 4 * (lane & 31);
  if (n >= k) return;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = m0 + wv * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
    if (m < M) {
      const float sc = sx * w_scale[m];
      const float4 v = make_float4((float)acc[0][r] * sc, (float)acc[1][r] * sc,
                                   (float)acc[2][r] * sc, (float)acc[3][r] * sc);
      *reinterpret_cast<float4 *>(yc + ((size_t)b * M + m) * k + n) = v;
    }
  }
}

// ---- plain fp32 FMA tile kernel (any storage types, any shape) ------------------------------------
template <int DT> struct WLoad;
template <> struct WLoad<WCC_F32> {
  static __device__ __forceinline__ float at(const void *w, size_t i) { return static_cast<const float *>(w)[i]; }
};
template <> struct WLoad<WCC_BF16> {
  static __device__ __forceinline__ float at(const void *w, size_t i) {
    return __uint_as_float((uint32_t) static_cast<const uint16_t *>(w)[i] << 16);
  }
};
template <> struct WLoad<WCC_I8> {
  static __device__ __forceinline__ float at(const void *w, size_t i) { return (float)static_cast<const int8_t *>(w)[i]; }
};

constexpr int FT = 64, FK = 16;

// grid = (ceil(k/64), ceil(M/64), B), block = 256; thread (ty, tx) computes rows ty*4..+3 and
// columns tx, tx+16, tx+32, tx+48 of the tile; channels are accumulated in increasing order.
// XM: 0 = fp32 activations as they are, 1 = int8 codes, 2 = fp32 activations quantised on load
template <int WDT, int XM>
__global__ __launch_bounds__(256) void pointwise_fma_kernel(const void *__restrict__ w,
                                                            const float *__restrict__ w_scale,
                                                            const void *__restrict__ xc,
                                                            const float *__restrict__ alpha,
                                                            bool slots, float *alpha_out,
                                                            float *__restrict__ yc, int M, int K,
                                                            int64_t k) {
  __shared__ float Ws[FK][FT + 1];
  __shared__ float Xs[FK][FT];
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int b = blockIdx.z, m0 = blockIdx.y * FT;
  const int64_t n0 = (int64_t)blockIdx.x * FT;
  float acc[4][4] = {};
  const float al = XM != 0 ? load_alpha(alpha, slots, alpha_out) : 0.f;
  for (int k0 = 0; k0 < K; k0 += FK) {
    // Ws[kk][mm] = w[m0 + mm][k0 + kk]
    for (int e = t; e < FT * FK; e += 256) {
      const int mm = e / FK, kk = e % FK;
      float v = 0.f;
      if (m0 + mm < M && k0 + kk < K) v = WLoad<WDT>::at(w, (size_t)(m0 + mm) * K + k0 + kk);
      Ws[kk][mm] = v;
    }
    for (int e = t; e < FT * FK; e += 256) {
      const int kk = e / FT, nn = e % FT;
      float v = 0.f;
      if (k0 + kk < K && n0 + nn < k) {
        const size_t at = ((size_t)b * K + k0 + kk) * k + n0 + nn;
        if (XM == 1) v = (float)static_cast<const int8_t *>(xc)[at];
        else if (XM == 2) v = (float)quant_code(static_cast<const float *>(xc)[at], al);
        else v = static_cast<const float *>(xc)[at];
      }
      Xs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FK; ++kk) {
      float a[4], x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = Ws[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) x[j] = Xs[kk][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], x[j], acc[i][j]);
    }
    __syncthreads();
  }
  const float sx = XM != 0 ? al / 127.f : 1.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
    const float sc = sx * (WDT == WCC_I8 ? w_scale[m] : 1.f);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t n = n0 + tx + 16 * j;
      if (n < k) yc[((size_t)b * M + m) * k + n] = acc[i][j] * sc;
    }
  }
}

template <int WDT, int XM>
hipError_t fma_launch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                      const void *xc, const float *alpha, bool slots, float *alpha_out, float *yc,
                      hipStream_t s) {
  dim3 grid((unsigned)((k + FT - 1) / FT), (d.C_out + FT - 1) / FT, d.B);
  hipLaunchKernelGGL((pointwise_fma_kernel<WDT, XM>), grid, dim3(256), 0, s, w, w_scale, xc, alpha,
                     slots, alpha_out, yc, d.C_out, d.C_in, k);
  return hipGetLastError();
}

template <int WDT>
hipError_t fma_dispatch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                        const void *xc, int xm, const float *alpha, bool slots, float *alpha_out,
                        float *yc, hipStream_t s) {
  switch (xm) {
    case 0: return fma_launch<WDT, 0>(d, k, w, w_scale, xc, alpha, slots, alpha_out, yc, s);
    case 1: return fma_launch<WDT, 1>(d, k, w, w_scale, xc, alpha, slots, alpha_out, yc, s);
    default: return fma_launch<WDT, 2>(d, k, w, w_scale, xc, alpha, slots, alpha_out, yc, s);
  }
}

}  // namespace

hipError_t launch_pointwise(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                            const void *xc, bool xc_is_f32, const float *alpha, bool slots,
                            float *alpha_out, float *yc, hipStream_t s) {
  const bool quant = d.act_quant_bits == 8;
  const int M = d.C_out, K = d.C_in;
  dim3 grid((unsigned)((k + BN - 1) / BN), (M + BM - 1) / BM, d.B);
  if (quant && d.w_dtype == WCC_BF16 && K % 8 == 0 && k % 4 == 0) {
    const uint16_t *wb = static_cast<const uint16_t *>(w);
    if (xc_is_f32)
      hipLaunchKernelGGL(pointwise_bf16_kernel<true>, grid, dim3(256), 0, s, wb, xc, alpha, slots, alpha_out, yc, M, K, k);
    else
      hipLaunchKernelGGL(pointwise_bf16_kernel<false>, grid, dim3(256), 0, s, wb, xc, alpha, slots, alpha_out, yc, M, K, k);
    return hipGetLastError();
  }
  if (quant && d.w_dtype == WCC_I8 && K % 16 == 0 && k % 4 == 0) {
    const int8_t *wi = static_cast<const int8_t *>(w);
    if (xc_is_f32)
      hipLaunchKernelGGL(pointwise_i8_kernel<true>, grid, dim3(256), 0, s, wi, w_scale, xc, alpha, slots, alpha_out, yc, M, K, k);
    else
      hipLaunchKernelGGL(pointwise_i8_kernel<false>, grid, dim3(256), 0, s, wi, w_scale, xc, alpha, slots, alpha_out, yc, M, K, k);
    return hipGetLastError();
  }
  const int xm = !quant ? 0 : (xc_is_f32 ? 2 : 1);
  switch (d.w_dtype) {
    case WCC_F32: return fma_dispatch<WCC_F32>(d, k, w, w_scale, xc, xm, alpha, slots, alpha_out, yc, s);
    case WCC_BF16: return fma_dispatch<WCC_BF16>(d, k, w, w_scale, xc, xm, alpha, slots, alpha_out, yc, s);
    case WCC_I8: return fma_dispatch<WCC_I8>(d, k, w, w_scale, xc, xm, alpha, slots, alpha_out, yc, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace wcc
