// Internal declarations shared by the translation units of libwcc (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wcc.h"

namespace wcc {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kMaxLevels = 4;      // register-resident strip transform up to 16 rows per lane
constexpr int kRadixBins = 2048;   // 11 + 11 + 10 bit radix select
constexpr int kSelectChunk = 4096; // keys per workgroup in the select kernels

// Geometry of the wavelet vector of one plane (Eq. wavelet_transform for d levels).
struct Geo {
  int H, W, d;
  int64_t N;
  __host__ __device__ int64_t n(int l) const { return (int64_t)(H >> l) * (W >> l); }
  // offset of band j (0 = y1, only for l = d; 1..3 = y2..y4) of level l
  __host__ __device__ int64_t band(int l, int j) const { return (int64_t)j * n(l); }
};

// How the workspace is carved up for one layer (offsets in bytes, all multiples of 256).
struct WsLayout {
  size_t norm_part;   // [G, B, N] fp32 partial channel norms
  size_t norm;        // [B, N] fp32
  size_t hist;        // [B, 3, kRadixBins] u32 + per-sample select state
  size_t state;       // [B] SelectState
  size_t blockcnt;    // [B, nblk] u32 x2 (gt, eq)
  size_t jmap;        // [B, N] int32: rank of a kept position, -1 otherwise
  size_t idx;         // [B, k] int32
  size_t alpha;       // 64 floats (alpha bits at [0])
  size_t coef;        // [B, C_in, N] fp32   (wcc_forward only)
  size_t xc32;        // [B, C_in, k] fp32
  size_t xq;          // [B, C_in, k] int8
  size_t yc;          // [B, C_out, k] fp32  (wcc_forward only)
  size_t total;
  int G;              // channel groups of the forward transform
  int nblk;           // select workgroups per sample
};

struct SelectState {
  uint32_t prefix;   // key bits fixed so far (high bits)
  uint32_t remain;   // how many more keys to take at or below this prefix
  uint32_t done[3];  // workgroups finished per pass ("last one picks")
  uint32_t pad[3];
};

WsLayout ws_layout(const wcc_desc &d);
int forward_groups(const wcc_desc &d);

// launchers (each returns hipGetLastError() after its launches)
hipError_t launch_haar_fwd(const wcc_desc &d, const float *x, float *coef, float *norm_part,
                           int G, hipStream_t s);
hipError_t launch_norm_reduce(const float *norm_part, int G, int64_t BN, float *norm, hipStream_t s);
hipError_t launch_channel_norm(const float *coef, int B, int C, int64_t N, float *norm, hipStream_t s);
hipError_t launch_select(const wcc_desc &d, const float *norm, int64_t k, void *ws_base,
                         const WsLayout &L, int32_t *idx, int32_t *jmap /*nullable*/, hipStream_t s);
hipError_t launch_jmap_from_idx(const int32_t *idx, int B, int64_t N, int64_t k, int32_t *jmap,
                                hipStream_t s);
hipError_t launch_alpha_init(float *alpha, float alpha_in, hipStream_t s);
hipError_t launch_gather(const float *coef, const int32_t *idx, int B, int C, int64_t N, int64_t k,
                         float *xc, float *alpha_max /*nullable: no max*/, hipStream_t s);
hipError_t launch_quantize(const float *xc32, int64_t n, const float *alpha, int8_t *codes,
                           hipStream_t s);
hipError_t launch_copy_f32(const float *src, float *dst, int64_t n, hipStream_t s);
hipError_t launch_pointwise(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                            const void *xc, const float *alpha, float *yc, hipStream_t s);
hipError_t launch_scatter_ihaar(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap,
                                float *y, hipStream_t s);

}  // namespace wcc
