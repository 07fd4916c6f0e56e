// Internal declarations shared by the translation units of libwcc (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>

#include "wcc.h"

namespace wcc {

constexpr int kWave = 64;          // CDNA wavefront width
using bf16_t = uint16_t;           // a bf16 bit pattern in memory
constexpr int kMaxLevels = 4;      // register-resident strip transform up to 16 rows per lane
constexpr int kRadixBins = 2048;   // 11 + 11 + 10 bit radix select
constexpr int kSelectChunk = 1024; // keys a select workgroup takes with one 16-byte load a thread
constexpr int kSfxStride = 1024;   // per-workgroup suffix sums of the low-digit histogram
constexpr int kAlphaSlots = 64;    // max|kept c| is reduced into this many slots, then combined
constexpr int kInvScratchBytes = 1024;  // one 16-byte line per lane for stores that must go nowhere

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
  size_t max_part;    // [G, B, N] fp32 largest |coefficient| of each channel group (8-bit layers)
  size_t norm;        // [B, N] fp32
  size_t hist;        // [B, 3, kRadixBins] u32
  size_t state;       // [B] SelectState
  size_t block_sfx;   // [B, nblk, kSfxStride] u16
  size_t block_gthi;  // [B, nblk] u32
  size_t jmap;        // [B, N] int32: rank of a kept position, -1 otherwise
  size_t idx;         // [B, k] int32
  size_t alpha;       // kAlphaSlots floats: partial maxima of |kept coefficient|
  size_t block_top;   // [B, nblk] fp32: the same, one per workgroup of the selection's last kernel
  size_t scratch;     // kInvScratchBytes: sink for the stores of lanes outside the plane
  size_t xc32;        // [B, C_in, k] fp32, or int8 codes in its first quarter
  size_t yc;          // [B, C_out, k] fp32  (wcc_forward only)
  size_t w8;          // [C_out, C_in] int8: WCC_I4 weights widened (else empty)
  size_t total;
  int G;              // channel groups of the forward transform
  int nblk;           // select workgroups per sample
  int sel_slots;      // 16-byte loads per thread in the select kernels: 1, 2 or 4
};

struct SelectState {
  uint32_t prefix[3];  // key bits fixed after pass 0, 1, 2 (prefix[2] is the threshold key)
  uint32_t remain[3];  // rank still to be resolved inside that prefix
  uint32_t pad[2];
};

// Per-call state that has to be cleared before the select passes run.  The forward
// transform's kernel does it on the side (one workgroup per sample) so that the fused path
// needs no separate clearing launch.
struct SelectPrep {
  uint32_t *hist;   // [B, 3, kRadixBins]; nullptr: nothing to prepare
  float *alpha;     // kAlphaSlots floats or nullptr
  float alpha_in;
};

__device__ inline void prep_sample(const SelectPrep &p, int b, int tid, int nthreads) {
  if (p.hist == nullptr) return;
  uint32_t *h = p.hist + (size_t)b * 3 * kRadixBins;
  for (int i = tid; i < 3 * kRadixBins; i += nthreads) h[i] = 0;
  if (b == 0 && p.alpha && tid < kAlphaSlots) p.alpha[tid] = p.alpha_in > 0.f ? p.alpha_in : 0.f;
}

// alpha = the largest of n partial maxima (n = 1: alpha itself; kAlphaSlots: the slots the
// second transform pass raised, or that hold the caller's alpha; otherwise one value per
// workgroup of the selection's last kernel).  Called by every thread of a workgroup of whole
// waves (at most 16); every thread gets the result.  Partial maxima are >= 0.
__device__ __forceinline__ float alpha_max(const float *__restrict__ p, int n) {
  __shared__ float wave_top[16];
  float v = 0.f;
  for (int i = threadIdx.x; i < n; i += blockDim.x) v = fmaxf(v, p[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  if ((threadIdx.x & (kWave - 1)) == 0) wave_top[threadIdx.x >> 6] = v;
  __syncthreads();
  float a = 0.f;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) a = fmaxf(a, wave_top[i]);
  return a;
}

// The scale-clip-round of Eq. (quantweights), signed, b = 8, operation by operation in fp32:
// u = v / alpha (correctly rounded); clip to [-1, 1]; level = round_half_even(127 * u).
// alpha <= 0 gives level 0.
//
// The division is the hot part (one per kept coefficient).  With y = RN(1/alpha) computed once,
// q0 = v*y, r = fma(-q0, alpha, v), q = fma(r, y, q0) is the correctly rounded quotient
// (Markstein's division theorem) unless alpha's significand is all ones; that case, and alpha
// outside [2^-60, 2^60] (where r could underflow for a v that still matters), take the IEEE
// divide.  Quotients too small to matter (|v| < alpha * 2^-9) round to level 0 either way.
struct Quant {
  float alpha, y;
  bool on, fast;
  // alpha is the same in every lane; reading it into a scalar register lets the compiler see
  // that (otherwise each level() becomes a divergent branch)
  __device__ __forceinline__ explicit Quant(float a)
      : alpha(__uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(a)))), y(0.f) {
    on = alpha > 0.f;
    fast = false;
    if (on) {
      y = __fdiv_rn(1.f, alpha);
      const uint32_t bits = __float_as_uint(alpha);
      fast = (bits & 0x7FFFFFu) != 0x7FFFFFu && alpha >= 0x1p-60f && alpha <= 0x1p60f;
    }
  }
  // the code as a float holding an integer in [-127, 127]; FAST: the caller has checked `fast`
  template <bool FAST>
  __device__ __forceinline__ float level_as(float v) const {
    float u;
    if constexpr (FAST) {
      // (a first quotient beyond +-2 clips to +-1 whatever the correction adds; held at +-2 it
      // cannot overflow, and with it the correction cannot turn infinity into NaN for a large
      // |v| over a small caller-supplied alpha)
      const float q0 = __builtin_amdgcn_fmed3f(__fmul_rn(v, y), -2.f, 2.f);
      const float r = __fmaf_rn(-q0, alpha, v);
      u = __fmaf_rn(r, y, q0);
    } else {
      u = __fdiv_rn(v, alpha);  // (alpha <= 0: whatever this gives is dropped below, no branch)
    }
    u = fminf(fmaxf(u, -1.f), 1.f);
    const float lv = rintf(__fmul_rn(127.f, u));
    return (FAST || on) ? lv : 0.f;
  }
  __device__ __forceinline__ float level(float v) const {
    return fast ? level_as<true>(v) : level_as<false>(v);
  }
  __device__ __forceinline__ int code(float v) const { return (int)level(v); }
};

// What stands in front of a layer's transform passes.
enum Front {
  kFrontNone = 0,   // the layer's input is x as it is
  kFrontDw = 1,     // K_dw x, convolved on the fly by both passes
  kFrontChain = 2   // K_dw iHWT(T^T Y_wt) of a producer layer, rebuilt from its compressed output
};
WsLayout ws_layout(const wcc_desc &d, int front = kFrontNone);
int forward_groups(const wcc_desc &d, int front);

// A producer layer's compressed output: t1 = iHWT(T^T yc), yc [B, C, k], jmap [B, N] its rank map
struct ChainSrc {
  const float *yc;
  const int32_t *jmap;
  int64_t k;
};
bool chain_supported(const wcc_desc &d);
// the two transform passes of a layer whose input is K_dw t1 (wdw [C_in, 3, 3]); otherwise as
// launch_haar_norm / launch_haar_keep
hipError_t launch_chain_norm(const wcc_desc &d, const ChainSrc &src, const float *wdw,
                             float *norm_part, float *max_part, int G, const SelectPrep &prep,
                             hipStream_t s);
hipError_t launch_chain_keep(const wcc_desc &d, int64_t k, const ChainSrc &src, const float *wdw,
                             const int32_t *jmap, void *xc, float *alpha_slots, float q_alpha,
                             const float *alpha_src, int n_alpha, float *alpha_pub, hipStream_t s);

// launchers (each returns hipGetLastError() after its launches)
hipError_t launch_haar_fwd(const wcc_desc &d, const float *x, float *coef, float *norm_part,
                           int G, const SelectPrep &prep, hipStream_t s);
// norm-only pass (no coefficient is written) and keep-only pass of the fused layer
// wdw (nullable, [C_in, 3, 3]): the transform's input is the depthwise 3x3 convolution of x
// with these kernels, computed on the fly; needs W % 4 == 0
// (x: fp32, or bf16 if d.act_dtype says so; the same for y and residual further down)
// max_part (nullable, [G, B, N]): also receives every group's largest |coefficient| per position
hipError_t launch_haar_norm(const wcc_desc &d, const void *x, float *norm_part, float *max_part,
                            int G, const SelectPrep &prep, const float *wdw, hipStream_t s);
// q_alpha > 0, or alpha_src given (n_alpha floats whose largest is the clipping parameter,
// read on the device): xc is int8 codes for that clipping parameter (alpha_slots unused); else
// xc is fp32 and alpha_slots (nullable) is raised to max |kept coefficient|
hipError_t launch_haar_keep(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap,
                            void *xc, float *alpha_slots /*nullable*/, const float *wdw /*nullable*/,
                            float q_alpha, const float *alpha_src /*nullable*/, int n_alpha,
                            float *alpha_pub /*nullable: receives that largest value*/,
                            hipStream_t s);
hipError_t launch_norm_reduce(const float *norm_part, int G, int64_t BN, float *norm, hipStream_t s);
hipError_t launch_channel_norm(const float *coef, int B, int C, int64_t N, bool squares, float *norm,
                               hipStream_t s);
SelectPrep make_prep(void *ws_base, const WsLayout &L, float *alpha_slots, float alpha_in);
hipError_t launch_select_init(const SelectPrep &p, int B, hipStream_t s);
// G > 1: norm_or_part is [G, B, N] partial norms, reduced into norm_out on the fly;
// G == 1: norm_or_part is the norm array and norm_out is unused.  Needs prepared state.
// top_part (nullable, [G, B, N], the max_part of launch_haar_norm): every workgroup of the last
// kernel writes the largest of its values over the positions it keeps to block_top
// (select_top_count() floats); the largest of those is max |kept coefficient|.  Plain stores:
// thousands of atomics arriving together on a few addresses serialise (25 us on 2048 of them).
// Group 0's plane of top_part may be overwritten with the maxima over the groups.
hipError_t launch_select(const wcc_desc &d, const float *norm_or_part, int G, float *norm_out,
                         int64_t k, void *ws_base, const WsLayout &L, int32_t *idx,
                         int32_t *jmap /*nullable*/, float *top_part, float *block_top,
                         hipStream_t s);
int select_top_count(const wcc_desc &d, const WsLayout &L);
hipError_t launch_jmap_from_idx(const int32_t *idx, int B, int64_t N, int64_t k, int32_t *jmap,
                                hipStream_t s);
// rank map (and index list, nullable) of "the first k positions of every sample"
hipError_t launch_jmap_prefix(int B, int64_t N, int64_t k, int32_t *jmap, int32_t *idx, hipStream_t s);
hipError_t launch_alpha_init(float *alpha_slots, float alpha_in, hipStream_t s);
// alpha_slots nullable: no maximum is taken
hipError_t launch_gather(const float *coef, const int32_t *idx, int B, int C, int64_t N, int64_t k,
                         float *xc, float *alpha_slots, hipStream_t s);
// codes = q(xc32) with alpha = max(slots); also writes alpha to alpha_out[0]
hipError_t launch_quantize(const float *xc32, int64_t n, const float *alpha_slots, float *alpha_out,
                           int8_t *codes, hipStream_t s);
// xc_is_f32 with act_quant_bits = 8: xc holds the unquantised kept coefficients and the
// kernel quantises them while loading (the fused path); otherwise xc is what the ABI says.
// alpha points at n_alpha partial maxima whose largest is the clipping parameter (combined in
// the kernel, and written to alpha_out[0] if that is not null); n_alpha = 1: alpha itself.
hipError_t launch_pointwise(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                            const void *xc, bool xc_is_f32, const float *alpha, int n_alpha,
                            float *alpha_out, float *yc, hipStream_t s);
// scratch: kInvScratchBytes of device memory that the kernel may overwrite with anything
// residual (nullable): [B, C_out, H, W] added to the result (may be y itself)
hipError_t launch_scatter_ihaar(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap,
                                void *y, float *scratch, const void *residual, hipStream_t s);
// out[i] = the two signed 4-bit codes of packed[i / 2] widened to int8 (n = number of codes, even)
hipError_t launch_unpack_i4(const uint8_t *packed, int8_t *out, int64_t n, hipStream_t s);
// depthwise 3x3, stride 1, zero padding 1: x, y [B, C, H, W], w [C, 3, 3]
hipError_t launch_depthwise3x3(int B, int C, int H, int W, const float *x, const float *w, float *y,
                               hipStream_t s);

}  // namespace wcc
