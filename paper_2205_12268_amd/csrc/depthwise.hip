// Depthwise 3x3 convolution, the K_dw between the two 1x1 convolutions of the inverted residual
// block (appendix "Inference times", Eq. (inverted)): cross-correlation, stride 1, zero padding
// 1, no bias, fp32.  y[b,c,r,q] = sum_{i,j} w[c][i][j] x[b,c,r+i-1,q+j-1].
//
// HBM-bound (one read and one write of the expanded tensor, the largest of the block).  A lane
// owns 4 adjacent columns (16-byte loads and stores, a wave covers 1 KiB-contiguous row
// segments) and walks kRows output rows with the three input rows it needs in registers; the
// two columns outside its four come from the neighbouring lanes' loads through a lane shuffle,
// and from memory only at the two ends of the wave's segment.  All kRows + 2 row loads of a
// lane go out before the first product.
#include "wcc_internal.h"

namespace wcc {
namespace {

constexpr int kRows = 8;  // output rows per lane

struct Row6 { float l; float4 m; float r; };  // columns q-1 | q..q+3 | q+4

// grid = (ceil(ceil(W/256) * ceil(H/kRows) / 4), C, B), block = 256 (a wave per strip segment).
// Needs W % 4 == 0.
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const float *__restrict__ x,
                                                          const float *__restrict__ w,
                                                          float *__restrict__ y, int C, int H, int W) {
  const int lane = threadIdx.x & 63;
  const int segs = (W + 255) / 256;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int seg = unit % segs, strip = unit / segs;
  const int c = blockIdx.y, b = blockIdx.z;
  const int q = seg * 256 + lane * 4, r0 = strip * kRows;
  if (r0 >= H) return;  // whole waves leave
  const bool in = q < W;
  const size_t plane = ((size_t)b * C + c) * (size_t)H * W;
  const float *xp = x + plane;
  float k[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) k[i] = w[(size_t)c * 9 + i];

  // rows r0-1 .. r0+kRows; rows outside the plane are zero
  Row6 row[kRows + 2];
#pragma unroll
  for (int i = 0; i < kRows + 2; ++i) {
    const int r = r0 - 1 + i;
    row[i].m = make_float4(0.f, 0.f, 0.f, 0.f);
    row[i].l = row[i].r = 0.f;
    const bool rin = r >= 0 && r < H;
    if (rin && in) row[i].m = *reinterpret_cast<const float4 *>(xp + (size_t)r * W + q);
    // the wave's ends: one lane each fetches the column beyond the segment
    if (rin && in && lane == 0 && q > 0) row[i].l = xp[(size_t)r * W + q - 1];
    if (rin && in && (lane == 63 || q + 4 >= W) && q + 4 < W) row[i].r = xp[(size_t)r * W + q + 4];
  }
#pragma unroll
  for (int i = 0; i < kRows + 2; ++i) {
    const float from_left = __shfl_up(row[i].m.w, 1, 64);     // lane-1's last column
    const float from_right = __shfl_down(row[i].m.x, 1, 64);  // lane+1's first column
    if (lane != 0) row[i].l = from_left;
    if (lane != 63 && q + 4 < W) row[i].r = from_right;
  }
  if (!in) return;
#pragma unroll
  for (int o = 0; o < kRows; ++o) {
    const int r = r0 + o;
    if (r >= H) break;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const Row6 &t = row[o + i];
      const float v[6] = {t.l, t.m.x, t.m.y, t.m.z, t.m.w, t.r};
#pragma unroll
      for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaf(k[i * 3 + j], v[e + j], acc[e]);
    }
    *reinterpret_cast<float4 *>(y + plane + (size_t)r * W + q) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  }
}

// any width: one thread per pixel
__global__ __launch_bounds__(256) void depthwise3x3_plain_kernel(const float *__restrict__ x,
                                                                 const float *__restrict__ w,
                                                                 float *__restrict__ y, int C, int H,
                                                                 int W) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int c = blockIdx.y, b = blockIdx.z;
  if (i >= (int64_t)H * W) return;
  const int r = (int)(i / W), q = (int)(i % W);
  const size_t plane = ((size_t)b * C + c) * (size_t)H * W;
  float acc = 0.f;
#pragma unroll
  for (int di = 0; di < 3; ++di)
#pragma unroll
    for (int dj = 0; dj < 3; ++dj) {
      const int rr = r + di - 1, qq = q + dj - 1;
      if (rr >= 0 && rr < H && qq >= 0 && qq < W)
        acc = fmaf(w[(size_t)c * 9 + di * 3 + dj], x[plane + (size_t)rr * W + qq], acc);
    }
  y[plane + i] = acc;
}

}  // namespace

hipError_t launch_depthwise3x3(int B, int C, int H, int W, const float *x, const float *w, float *y,
                               hipStream_t s) {
  if (W % 4 == 0) {
    const unsigned units = (unsigned)(((W + 255) / 256) * ((H + kRows - 1) / kRows));
    hipLaunchKernelGGL(depthwise3x3_kernel, dim3((units + 3) / 4, C, B), dim3(256), 0, s, x, w, y, C, H, W);
  } else {
    const unsigned gx = (unsigned)(((int64_t)H * W + 255) / 256);
    hipLaunchKernelGGL(depthwise3x3_plain_kernel, dim3(gx, C, B), dim3(256), 0, s, x, w, y, C, H, W);
  }
  return hipGetLastError();
}

}  // namespace wcc
