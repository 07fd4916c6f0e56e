// Joint shrinkage (Alg. 1: the index set I holds the k = ceil(gamma n_w n_h) positions whose
// channel vectors have the largest norm):
// per sample, the k largest of N non-negative fp32 norms, ties toward the lower position,
// emitted in ascending position order.
//
// Design.  Non-negative floats order like their bit patterns, so the k-th largest norm is
// found exactly by a most-significant-digit radix select on uint32 keys: three histogram
// passes (11 + 11 + 10 bits) spread over many workgroups per sample, integer atomics only.
// Every workgroup of the NEXT kernel turns the finished histogram of the previous pass into
// the digit to descend into by itself (an 8 KiB read and one block scan): no workgroup waits
// for another and no device-wide fence is needed -- on this chip such a fence writes back a
// whole L2, which costs more than the pass.  The third pass also leaves, per workgroup, the
// suffix sums of its own low-digit histogram; once the threshold key T is known they give every workgroup's count of keys
// above T and equal to T without another pass over the keys.  The last kernel is an ordered
// compaction: a position is kept if key > T, or key == T and fewer than r equal keys precede
// it (r = how many keys equal to T are still needed).  Ordering comes from prefix sums,
// never from the arrival order of atomics, so the result is the same on every run.
// The first pass can take the channel-group partial norms of the forward transform and
// reduce them on the fly (fixed order), writing the final norms as a by-product.
#include "wcc_internal.h"

namespace wcc {
namespace {

constexpr int kThreads = 256;                  // 4 waves
constexpr int kWaves = kThreads / 64;
constexpr int kPer = kSelectChunk / kThreads;  // 4 keys per thread
static_assert(kPer == 4, "one 16-byte load per thread");

__device__ __forceinline__ uint32_t digit_of(uint32_t key, int pass) {
  return pass == 0 ? key >> 21 : pass == 1 ? (key >> 10) & 0x7FFu : key & 0x3FFu;
}
// keys whose bits above the current digit equal those of `prefix`
__device__ __forceinline__ bool matches(uint32_t key, uint32_t prefix, int pass) {
  return pass == 0 ? true : pass == 1 ? (key >> 21) == (prefix >> 21) : (key >> 10) == (prefix >> 10);
}

// lh[digit] += 1 for every valid lane; lanes of a wave that share a digit are counted by one
// LDS atomic (two leader rounds catch the big tie classes, the rest goes lane by lane)
__device__ __forceinline__ void hist_add(uint32_t *lh, uint32_t digit, bool valid) {
  const int lane = threadIdx.x & 63;
  uint64_t todo = __ballot(valid);
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if (todo == 0) break;
    const int leader = __ffsll((unsigned long long)todo) - 1;
    const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);  // leader is wave-uniform
    const uint64_t same = __ballot(valid && digit == d0);
    if (lane == leader) atomicAdd(&lh[d0], (uint32_t)__popcll(same));
    if (digit == d0) valid = false;
    todo &= ~same;
  }
  if (valid) atomicAdd(&lh[digit], 1u);
}

// The same for a workgroup whose digits are spread out: one round, the class of the first
// valid lane is counted by one atomic, every other lane adds for itself.
__device__ __forceinline__ void hist_add_spread(uint32_t *lh, uint32_t digit, bool valid) {
  if (valid) {
    const uint32_t d0 = __builtin_amdgcn_readfirstlane(digit);
    const uint64_t same = __ballot(digit == d0);
    const int first = __ffsll((unsigned long long)same) - 1;
    const uint32_t val = digit != d0 ? 1u : ((int)(threadIdx.x & 63) == first ? (uint32_t)__popcll(same) : 0u);
    if (val) atomicAdd(&lh[digit], val);
  }
}

// Inclusive prefix sum over the 64 lanes of a wave (all of them active), on the data-parallel
// shifts of the vector unit instead of six round trips through the LDS crossbar: shifts by
// 1, 2, 4, 8 inside rows of 16 lanes (a lane shifted in from outside its row adds 0), then lane
// 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
  uint32_t v = x;
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31
  return v;
}

// Smallest / largest value over the 64 lanes (all active), every lane gets it: the moves of the
// scan with the operation's identity shifted in; lane 63 ends up with the whole wave's result.
template <bool MAX>
__device__ __forceinline__ uint32_t wave_extreme(uint32_t x) {
  constexpr int id = MAX ? 0 : -1;
  uint32_t v = x;
  auto join = [](uint32_t a, uint32_t b) { return MAX ? max(a, b) : min(a, b); };
  v = join(v, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)v, 0x111, 0xf, 0xf, false));
  v = join(v, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)v, 0x112, 0xf, 0xf, false));
  v = join(v, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)v, 0x114, 0xf, 0xf, false));
  v = join(v, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)v, 0x118, 0xf, 0xf, false));
  v = join(v, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)v, 0x142, 0xa, 0xf, false));
  v = join(v, (uint32_t)__builtin_amdgcn_update_dpp(id, (int)v, 0x143, 0xc, 0xf, false));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// block-wide sum of v (all threads get it); `tmp` has NW (waves per workgroup) entries
template <int NW = kWaves>
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *tmp) {
  v = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_scan(v), 63);
  __syncthreads();  // tmp may still be read from a previous use
  if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = v;
  __syncthreads();
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) s += tmp[i];
  return s;
}

// block-wide exclusive scan in thread order; `tmp` has NW (waves per workgroup) entries
template <int NW = kWaves>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *tmp) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t inc = wave_inclusive_scan(v);
  __syncthreads();
  if (lane == 63) tmp[wv] = inc;
  __syncthreads();
  uint32_t before = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i)
    if (i < wv) before += tmp[i];
  return before + inc - v;
}

__global__ __launch_bounds__(256) void select_init_kernel(SelectPrep p, int B) {
  if ((int)blockIdx.x < B) prep_sample(p, blockIdx.x, threadIdx.x, blockDim.x);
}

// Four keys of this thread.  REDUCE: keys are sums of G partial-norm planes (added in
// increasing group order), and the sums are written to norm.
template <bool REDUCE>
__device__ __forceinline__ uint4 load_keys(const float *__restrict__ src, float *__restrict__ norm,
                                           int G, int64_t BN, int64_t at) {
  float4 v = *reinterpret_cast<const float4 *>(src + at);
  if constexpr (REDUCE) {
    int g = 1;
    for (; g + 4 <= G; g += 4) {  // four loads in flight, added in increasing group order
      float4 t[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) t[i] = *reinterpret_cast<const float4 *>(src + (int64_t)(g + i) * BN + at);
#pragma unroll
      for (int i = 0; i < 4; ++i) { v.x += t[i].x; v.y += t[i].y; v.z += t[i].z; v.w += t[i].w; }
    }
    for (; g < G; ++g) {
      const float4 t = *reinterpret_cast<const float4 *>(src + (int64_t)g * BN + at);
      v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
    *reinterpret_cast<float4 *>(norm + at) = v;
  }
  return make_uint4(__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z),
                    __float_as_uint(v.w));
}

// max over the G channel groups of their largest |coefficient| at this thread's four positions
// (top_part [G, B, N], written by the norm-only transform pass)
__device__ __forceinline__ float4 load_top(const float *__restrict__ top_part, int G, int64_t BN,
                                           int64_t at) {
  float4 m = *reinterpret_cast<const float4 *>(top_part + at);
  int g = 1;
  for (; g + 4 <= G; g += 4) {  // four loads in flight
    float4 t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = *reinterpret_cast<const float4 *>(top_part + (int64_t)(g + i) * BN + at);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      m.x = fmaxf(m.x, t[i].x); m.y = fmaxf(m.y, t[i].y); m.z = fmaxf(m.z, t[i].z); m.w = fmaxf(m.w, t[i].w);
    }
  }
  for (; g < G; ++g) {
    const float4 t = *reinterpret_cast<const float4 *>(top_part + (int64_t)g * BN + at);
    m.x = fmaxf(m.x, t.x); m.y = fmaxf(m.y, t.y); m.z = fmaxf(m.z, t.z); m.w = fmaxf(m.w, t.w);
  }
  return m;
}

// block_top[slot] = the workgroup's largest kept |coefficient| (v >= 0 in every thread, all
// threads of the workgroup call; `tmp` has NW entries).  A plain store per workgroup: the
// consumers take the maximum over all of them.
template <int NW>
__device__ __forceinline__ void publish_top(float v, float *block_top, size_t slot, uint32_t *tmp) {
  const uint32_t w = wave_extreme<true>(__float_as_uint(v));  // (>= 0: floats order like their bits)
  __syncthreads();  // tmp may still be read from a previous use
  if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = w;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) mine = max(mine, tmp[i]);
    block_top[slot] = __uint_as_float(mine);
  }
}

// Turns the finished histogram of pass P into the digit that holds the remaining rank:
// the digit D with count(> D) < remain <= count(>= D), scanning from the top digit down.
// Every thread returns the same (prefix, remain) for the next pass.
template <int P, int THREADS = kThreads>
__device__ __forceinline__ void pick_digit(const uint32_t *gh, uint32_t &prefix,
                                           uint32_t &remain, uint32_t *tmp, uint32_t *bcast) {
  constexpr int bins = P == 2 ? 1024 : kRadixBins;
  constexpr int per = bins / THREADS;  // consecutive digits per thread, from the top
  const int t = threadIdx.x;
  uint32_t cnt[per], sum = 0;
#pragma unroll
  for (int i = 0; i < per; ++i) {
    cnt[i] = gh[bins - 1 - (t * per + i)];
    sum += cnt[i];
  }
  uint32_t above = block_exclusive_scan<THREADS / 64>(sum, tmp);
#pragma unroll
  for (int i = 0; i < per; ++i) {
    if (above < remain && remain <= above + cnt[i]) {
      const uint32_t digit = bins - 1 - (t * per + i);
      bcast[0] = prefix | (P == 0 ? digit << 21 : P == 1 ? digit << 10 : digit);
      bcast[1] = remain - above;
    }
    above += cnt[i];
  }
  __syncthreads();
  prefix = bcast[0];
  remain = bcast[1];
  __syncthreads();
}

// (prefix, remain) after passes 0..UPTO-1: earlier picks come from the state (stored by a
// previous kernel), the newest one is computed here from the histogram that kernel finished.
template <int UPTO>
__device__ __forceinline__ void current_state(const uint32_t *hist_b, SelectState *s,
                                              uint32_t k, uint32_t &prefix, uint32_t &remain,
                                              uint32_t *tmp, uint32_t *bcast, bool store) {
  prefix = 0;
  remain = k;
  if constexpr (UPTO == 0) return;
  if constexpr (UPTO >= 2) {
    prefix = s->prefix[UPTO - 2];
    remain = s->remain[UPTO - 2];
  }
  if (threadIdx.x == 0) { bcast[0] = prefix; bcast[1] = remain; }  // rank beyond the data: unchanged
  __syncthreads();
  pick_digit<UPTO - 1>(hist_b + (size_t)(UPTO - 1) * kRadixBins, prefix, remain, tmp, bcast);
  if (store && threadIdx.x == 0) {
    s->prefix[UPTO - 1] = prefix;
    s->remain[UPTO - 1] = remain;
  }
}

// One histogram pass.  grid = (nblk, B), block = 256.
// PASS 0 with REDUCE reads partial norms `src` [G, B, N] and writes `norm`; otherwise src is
// the norm array itself.  PASS 2 also writes this workgroup's suffix sums and its count of
// keys above the 22-bit prefix.
// SLOTS: 16-byte loads per thread (a workgroup takes 1024 * SLOTS keys; slot s of thread t
// covers the four positions from (s * 256 + t) * 4 on inside the workgroup's chunk).
template <int PASS, bool REDUCE, int SLOTS>
__global__ __launch_bounds__(kThreads) void select_hist_kernel(const float *__restrict__ src,
                                                               float *__restrict__ norm, int G,
                                                               int64_t N, int B, uint32_t k,
                                                               uint32_t *hist, SelectState *st,
                                                               int nblk,
                                                               uint16_t *__restrict__ block_sfx,
                                                               uint32_t *__restrict__ block_gthi) {
  constexpr int bins = PASS == 2 ? 1024 : kRadixBins;
  __shared__ uint32_t lh[kRadixBins];
  __shared__ uint32_t tmp[kWaves];
  __shared__ uint32_t bcast[2];
  const int b = blockIdx.y, t = threadIdx.x;
  uint32_t *hist_b = hist + (size_t)b * 3 * kRadixBins;
  uint32_t *gh = hist_b + (size_t)PASS * kRadixBins;

  for (int i = t; i < bins; i += kThreads) lh[i] = 0;
  // the keys do not depend on the digit picked below: their load travels under it
  const int64_t q0 = (int64_t)blockIdx.x * (kSelectChunk * SLOTS) + (int64_t)t * kPer;
  uint4 k4[SLOTS];
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl) {
    const int64_t q = q0 + (int64_t)sl * kSelectChunk;
    k4[sl] = make_uint4(0, 0, 0, 0);  // N is a multiple of 4: a slot's four keys are all in or all out
    if (q < N) k4[sl] = load_keys<REDUCE>(src, norm, G, (int64_t)B * N, (int64_t)b * N + q);
  }
  uint32_t prefix, remain;
  current_state<PASS>(hist_b, st + b, k, prefix, remain, tmp, bcast, blockIdx.x == 0);
  __syncthreads();
  uint32_t above = 0;
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl) {
    const bool in = q0 + (int64_t)sl * kSelectChunk < N;
    const uint32_t key[4] = {k4[sl].x, k4[sl].y, k4[sl].z, k4[sl].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      hist_add(lh, digit_of(key[e], PASS), in && matches(key[e], prefix, PASS));
      if (PASS == 2) above += (in && (key[e] >> 10) > (prefix >> 10)) ? 1u : 0u;
    }
  }
  __syncthreads();
  for (int i = t; i < bins; i += kThreads) {
    const uint32_t v = lh[i];
    if (v) atomicAdd(&gh[i], v);
  }
  if constexpr (PASS == 2) {
    // sfx[d] = number of this workgroup's matching keys with low digit >= d
    constexpr int per = bins / kThreads;  // 4 digits per thread, from the top
    uint32_t c[per], sum = 0;
#pragma unroll
    for (int i = 0; i < per; ++i) {
      c[i] = lh[bins - 1 - (t * per + i)];
      sum += c[i];
    }
    uint32_t run = block_exclusive_scan(sum, tmp);
    const size_t blk = (size_t)b * nblk + blockIdx.x;
#pragma unroll
    for (int i = 0; i < per; ++i) {
      run += c[i];
      block_sfx[blk * kSfxStride + (bins - 1 - (t * per + i))] = (uint16_t)run;
    }
    const uint32_t tot_above = block_sum(above, tmp);
    if (t == 0) block_gthi[blk] = tot_above;
  }
}

// Ordered compaction.  grid = (nblk, B), block = 256.  jmap (nullable) gets the rank of
// every kept position and -1 for every dropped one.  top_part (nullable, [G, B, N]): the largest
// |coefficient| over the channels at every position; its maximum over the positions this
// workgroup keeps goes to block_top[b, blockIdx.x] (the largest of those is the layer's clipping
// parameter alpha).
template <int SLOTS>
__global__ __launch_bounds__(kThreads) void select_emit_kernel(const float *__restrict__ norm,
                                                               int64_t N, int64_t k,
                                                               const uint32_t *__restrict__ hist,
                                                               SelectState *st,
                                                               const uint16_t *__restrict__ block_sfx,
                                                               const uint32_t *__restrict__ block_gthi,
                                                               int nblk, int32_t *__restrict__ idx,
                                                               int32_t *__restrict__ jmap,
                                                               const float *__restrict__ top_part,
                                                               int G, int B, float *block_top) {
  __shared__ uint32_t tmp[kWaves];
  __shared__ uint32_t bcast[2];
  const int b = blockIdx.y, t = threadIdx.x;
  const uint32_t *keys = reinterpret_cast<const uint32_t *>(norm) + (size_t)b * N;
  // (the keys do not depend on the threshold: their load travels under its computation)
  const int64_t q0 = (int64_t)blockIdx.x * (kSelectChunk * SLOTS) + (int64_t)t * kPer;
  uint4 k4[SLOTS];
  float4 top4[SLOTS];
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl) {
    const int64_t q = q0 + (int64_t)sl * kSelectChunk;
    k4[sl] = make_uint4(0, 0, 0, 0);
    top4[sl] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (q < N) {
      k4[sl] = *reinterpret_cast<const uint4 *>(keys + q);
      if (top_part) top4[sl] = load_top(top_part, G, (int64_t)B * N, (int64_t)b * N + q);
    }
  }
  uint32_t T, r_take;  // threshold key, and how many keys equal to it are still needed
  current_state<3>(hist + (size_t)b * 3 * kRadixBins, st + b, (uint32_t)k, T, r_take, tmp, bcast,
                   blockIdx.x == 0);
  const uint32_t tlow = T & 0x3FFu;

  // keys above / equal to T in the workgroups before this one
  uint32_t gt0 = 0, eq0 = 0;
  for (int i = t; i < (int)blockIdx.x; i += kThreads) {
    const size_t blk = (size_t)b * nblk + i;
    const uint32_t ge = block_sfx[blk * kSfxStride + tlow];
    const uint32_t gtl = tlow + 1 < 1024 ? block_sfx[blk * kSfxStride + tlow + 1] : 0u;
    gt0 += block_gthi[blk] + gtl;
    eq0 += ge - gtl;
  }
  gt0 = block_sum(gt0, tmp);
  eq0 = block_sum(eq0, tmp);

  // Position order inside the workgroup's chunk is slot by slot, thread by thread: one block
  // scan a slot, on top of the totals of the slots before it.  Counts are packed
  // hi16: keys above T, lo16: keys equal to T (each <= 4096 a workgroup).
  float kept_top = 0.f;
  int32_t *out = idx + (size_t)b * k;
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl) {
    const int64_t q = q0 + (int64_t)sl * kSelectChunk;
    const bool in = q < N;
    const uint32_t key[4] = {k4[sl].x, k4[sl].y, k4[sl].z, k4[sl].w};
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (in) packed += ((key[e] > T) << 16) + (key[e] == T);
    const uint32_t ex = block_exclusive_scan(packed, tmp);
    uint32_t gt = gt0 + (ex >> 16), eq = eq0 + (ex & 0xFFFFu);
    if (SLOTS > 1) {  // the slot's totals (tmp holds the waves' inclusive sums until the next scan)
      uint32_t tot = 0;
#pragma unroll
      for (int i = 0; i < kWaves; ++i) tot += tmp[i];
      gt0 += tot >> 16;
      eq0 += tot & 0xFFFFu;
    }
    if (in) {
      const float top[4] = {top4[sl].x, top4[sl].y, top4[sl].z, top4[sl].w};
      int32_t jm[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool is_gt = key[e] > T, is_eq = key[e] == T;
        const bool keep = is_gt || (is_eq && eq < r_take);
        const uint32_t j = gt + min(eq, r_take);
        if (keep) out[j] = (int32_t)(q + e);
        jm[e] = keep ? (int32_t)j : -1;
        kept_top = fmaxf(kept_top, keep ? top[e] : 0.f);
        gt += is_gt; eq += is_eq;
      }
      if (jmap) *reinterpret_cast<int4 *>(jmap + (size_t)b * N + q) = make_int4(jm[0], jm[1], jm[2], jm[3]);
    }
  }
  if (top_part)  // (uniform over the grid)
    publish_top<kWaves>(kept_top, block_top, (size_t)b * nblk + blockIdx.x, tmp);
}

// ---- small planes: the whole select of one sample in ONE workgroup -------------------------
// For N <= 16384 the four kernels above are launch gaps and little else.  Here one workgroup of
// 1024 threads holds all keys of a sample in registers (slot s of thread t covers the four
// positions from (s * 1024 + t) * 4 on: every load is one contiguous 16 KiB row), runs the
// digit passes on an LDS histogram and emits idx and jmap in position order.  Same result,
// bit for bit.
//
// With all keys in one place the digits need not be raw bit fields: the passes work on
// rel = key - min(keys), whose significant bits (those of max - min) are cut into fields of at
// most 11 bits from the top.  Norms of one plane share their upper exponent bits, so the raw
// top field would put nearly all keys into a handful of bins and the LDS atomics of the 16
// waves would serialise on them; the relative top field spreads them over the whole histogram.
// Passes whose field is empty are skipped.
constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / 64;
constexpr int kSmallSlots = 4;  // 16-byte loads per thread at most (beyond that the one
                                // workgroup is slower than the four spread-out kernels)
constexpr int64_t kSmallMaxN = (int64_t)4 * kSmallSlots * kSmallThreads;

// One pass over the field rel[hi-1 : lo] (hi - lo <= 11) of the keys that agree with `prefix`
// above bit hi (FIRST: no bit is set above hi, all keys take part); then the digit that holds
// the remaining rank is appended to prefix.
template <bool FIRST>
__device__ __forceinline__ void small_pass(const uint32_t (&rel)[4 * kSmallSlots], uint32_t vmask,
                                           int slots, int hi, int lo, uint32_t &prefix,
                                           uint32_t &remain, uint32_t *lh, uint32_t *tmp,
                                           uint32_t *bcast) {
  const int t = threadIdx.x;
  const uint32_t fmask = (1u << (hi - lo)) - 1u;
  for (int i = t; i < kRadixBins; i += kSmallThreads) lh[i] = 0;
  if (t == 0) { bcast[0] = prefix; bcast[1] = remain; }  // rank beyond the data: unchanged
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kSmallSlots; ++s) {
    if (s < slots) {  // uniform over the workgroup
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t r = rel[4 * s + e];
        bool agrees = true;
        if constexpr (!FIRST) agrees = (r >> hi) == (prefix >> hi);
        hist_add_spread(lh, (r >> lo) & fmask, ((vmask >> s) & 1u) && agrees);
      }
    }
  }
  __syncthreads();
  // two consecutive digits per thread, from the top
  uint32_t cnt[2], sum = 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    cnt[i] = lh[kRadixBins - 1 - (t * 2 + i)];
    sum += cnt[i];
  }
  uint32_t above = block_exclusive_scan<kSmallWaves>(sum, tmp);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (above < remain && remain <= above + cnt[i]) {
      const uint32_t digit = kRadixBins - 1 - (t * 2 + i);
      bcast[0] = prefix | (digit << lo);
      bcast[1] = remain - above;
    }
    above += cnt[i];
  }
  __syncthreads();
  prefix = bcast[0];
  remain = bcast[1];
  __syncthreads();
}

// The G partial planes of a small map summed (and their maxima taken) by the whole chip before
// the one-workgroup-a-sample kernel below: with many groups that kernel would otherwise read
// G x N values per sample through a single compute unit.  grid = (ceil(N / 1024), B), block = 256.
// The maxima land in group 0's plane of top_part (each position is read and written by one thread).
__global__ __launch_bounds__(256) void combine_parts_kernel(const float *__restrict__ part,
                                                            float *__restrict__ norm, int G, int64_t N,
                                                            int B, float *top_part) {
  const int64_t pos = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (pos >= N) return;
  const int64_t at = (int64_t)blockIdx.y * N + pos;
  load_keys<true>(part, norm, G, (int64_t)B * N, at);
  if (top_part) *reinterpret_cast<float4 *>(top_part + at) = load_top(top_part, G, (int64_t)B * N, at);
}

// The partial planes are combined first from this many groups and this many values a sample on
// (below that the extra launch costs more than the one workgroup's reads: the deep layers of the
// 16-layer stack have 2048-8192 positions in up to 32 groups)
constexpr int kCombineGroups = 4;
constexpr int64_t kCombineValues = 1 << 18;

// grid = B, block = 1024.  REDUCE as in load_keys.
template <bool REDUCE>
__global__ __launch_bounds__(kSmallThreads) void select_small_kernel(
    const float *__restrict__ src, float *__restrict__ norm, int G, int64_t N, int B, uint32_t k,
    int slots, int32_t *__restrict__ idx, int32_t *__restrict__ jmap,
    const float *__restrict__ top_part, float *block_top) {
  __shared__ uint32_t lh[kRadixBins];
  __shared__ uint32_t tmp[kSmallSlots * kSmallWaves];
  __shared__ uint32_t bcast[2];
  const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
  uint32_t rel[4 * kSmallSlots];
  float topv[4 * kSmallSlots];  // largest |coefficient| over the channels at the key's position
  uint32_t vmask = 0;  // bit s: slot s of this thread lies inside the plane (N is a multiple of 4)
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
  for (int s = 0; s < kSmallSlots; ++s) {
    const int64_t pos = ((int64_t)s * kSmallThreads + t) * 4;
    uint4 k4 = make_uint4(0, 0, 0, 0);
    float4 t4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s < slots && pos < N) {
      k4 = load_keys<REDUCE>(src, norm, G, (int64_t)B * N, (int64_t)b * N + pos);
      if (top_part) t4 = load_top(top_part, G, (int64_t)B * N, (int64_t)b * N + pos);
      vmask |= 1u << s;
      kmin = min(kmin, min(min(k4.x, k4.y), min(k4.z, k4.w)));
      kmax = max(kmax, max(max(k4.x, k4.y), max(k4.z, k4.w)));
    }
    rel[4 * s] = k4.x; rel[4 * s + 1] = k4.y; rel[4 * s + 2] = k4.z; rel[4 * s + 3] = k4.w;
    topv[4 * s] = t4.x; topv[4 * s + 1] = t4.y; topv[4 * s + 2] = t4.z; topv[4 * s + 3] = t4.w;
  }
  // smallest and largest key of the sample
  kmin = wave_extreme<false>(kmin);
  kmax = wave_extreme<true>(kmax);
  if (lane == 0) { tmp[wv] = kmin; tmp[kSmallWaves + wv] = kmax; }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSmallWaves; ++i) {
    kmin = min(kmin, tmp[i]);
    kmax = max(kmax, tmp[kSmallWaves + i]);
  }
#pragma unroll
  for (int i = 0; i < 4 * kSmallSlots; ++i) rel[i] -= kmin;  // slots outside the plane: unused
  const int nbits = 32 - __clz((int)(kmax - kmin));  // 0 when all keys are equal (clz(0) = 32)

  uint32_t T = 0, r_take = k;  // threshold (relative key) and how many keys equal to it to take
  const int lo0 = max(nbits - 11, 0), lo1 = max(nbits - 22, 0);
  small_pass<true>(rel, vmask, slots, nbits, lo0, T, r_take, lh, tmp, bcast);
  if (lo0 > 0) small_pass<false>(rel, vmask, slots, lo0, lo1, T, r_take, lh, tmp, bcast);
  if (lo1 > 0) small_pass<false>(rel, vmask, slots, lo1, 0, T, r_take, lh, tmp, bcast);

  // Ordered compaction as in select_emit_kernel.  Position order is slot-major, then thread,
  // then the four keys of a slot: a wave scan per slot, then a scan over the 64 (slot, wave)
  // totals.  Counts (above T | equal to T) are packed 16 + 16 bits: N <= 16384.
  uint32_t ex[kSmallSlots];
#pragma unroll
  for (int s = 0; s < kSmallSlots; ++s) {
    uint32_t packed = 0;
    if ((vmask >> s) & 1u) {
#pragma unroll
      for (int e = 0; e < 4; ++e) packed += ((rel[4 * s + e] > T) << 16) + (rel[4 * s + e] == T);
    }
    uint32_t inc = packed;
    if (s < slots) inc = wave_inclusive_scan(packed);  // (uniform over the workgroup)
    ex[s] = inc - packed;
    if (lane == 63) tmp[s * kSmallWaves + wv] = inc;
  }
  __syncthreads();
  static_assert(kSmallSlots * kSmallWaves == 64, "one wave scans the totals");
  if (t < 64) {  // wave 0: exclusive scan of the 64 totals
    const uint32_t v = tmp[t];
    tmp[t] = wave_inclusive_scan(v) - v;
  }
  __syncthreads();

  int32_t *out = idx + (size_t)b * k;
  float kept_top = 0.f;  // largest |coefficient| over the channels at a kept position
#pragma unroll
  for (int s = 0; s < kSmallSlots; ++s) {
    if ((vmask >> s) & 1u) {
      const int e0 = s * kSmallWaves + wv;
      const uint32_t before = tmp[e0] + ex[s];
      uint32_t gt = before >> 16, eq = before & 0xFFFFu;
      const int64_t pos = ((int64_t)s * kSmallThreads + t) * 4;
      int32_t jm[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t ky = rel[4 * s + e];
        const bool is_gt = ky > T, is_eq = ky == T;
        const bool keep = is_gt || (is_eq && eq < r_take);
        const uint32_t j = gt + min(eq, r_take);
        if (keep) out[j] = (int32_t)(pos + e);
        jm[e] = keep ? (int32_t)j : -1;
        kept_top = fmaxf(kept_top, keep ? topv[4 * s + e] : 0.f);
        gt += is_gt; eq += is_eq;
      }
      if (jmap) *reinterpret_cast<int4 *>(jmap + (size_t)b * N + pos) = make_int4(jm[0], jm[1], jm[2], jm[3]);
    }
  }
  if (top_part)  // (uniform over the grid)
    publish_top<kSmallWaves>(kept_top, block_top, (size_t)b, tmp);
}

// jmap from an arbitrary ascending index list: fill with -1, then jmap[b][idx[b][j]] = j
__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t *p, int64_t n, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ __launch_bounds__(256) void jmap_scatter_kernel(const int32_t *__restrict__ idx,
                                                           int64_t N, int64_t k,
                                                           int32_t *__restrict__ jmap) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (j >= k) return;
  const int32_t q = idx[(size_t)b * k + j];
  if (q >= 0 && q < N) jmap[(size_t)b * N + q] = (int32_t)j;
}

// the index list "first k positions" (coarsest bands first): jmap[b][q] = q < k ? q : -1,
// idx[b][j] = j (idx nullable)
__global__ __launch_bounds__(256) void jmap_prefix_kernel(int64_t N, int64_t k,
                                                          int32_t *__restrict__ jmap,
                                                          int32_t *__restrict__ idx) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (q >= N) return;
  jmap[(size_t)b * N + q] = q < k ? (int32_t)q : -1;
  if (idx && q < k) idx[(size_t)b * k + q] = (int32_t)q;
}

}  // namespace

hipError_t launch_jmap_prefix(int B, int64_t N, int64_t k, int32_t *jmap, int32_t *idx,
                              hipStream_t s) {
  hipLaunchKernelGGL(jmap_prefix_kernel, dim3((unsigned)((N + 255) / 256), B), dim3(256), 0, s, N, k,
                     jmap, idx);
  return hipGetLastError();
}

SelectPrep make_prep(void *ws_base, const WsLayout &L, float *alpha_slots, float alpha_in) {
  char *ws = static_cast<char *>(ws_base);
  SelectPrep p;
  p.hist = reinterpret_cast<uint32_t *>(ws + L.hist);
  p.alpha = alpha_slots;
  p.alpha_in = alpha_in;
  return p;
}

// how many partial maxima launch_select leaves in block_top: one per workgroup of its last kernel
int select_top_count(const wcc_desc &d, const WsLayout &L) {
  return (int64_t)d.H * d.W <= kSmallMaxN ? d.B : d.B * L.nblk;
}

hipError_t launch_select_init(const SelectPrep &p, int B, hipStream_t s) {
  hipLaunchKernelGGL(select_init_kernel, dim3(B), dim3(256), 0, s, p, B);
  return hipGetLastError();
}

// the three histogram passes and the compaction, SLOTS 16-byte loads a thread
template <int SLOTS>
static hipError_t launch_passes(const wcc_desc &d, const float *norm_or_part, int G, float *norm_out,
                                int64_t k, uint32_t *hist, SelectState *st, uint16_t *sfx,
                                uint32_t *gthi, int nblk, int32_t *idx, int32_t *jmap,
                                float *top_part, float *block_top, hipStream_t s) {
  const int64_t N = (int64_t)d.H * d.W;
  const uint32_t k32 = (uint32_t)k;
  dim3 grid(nblk, d.B), block(kThreads);
  const float *norm = norm_or_part;
  if (G > 1) {
    hipLaunchKernelGGL((select_hist_kernel<0, true, SLOTS>), grid, block, 0, s, norm_or_part, norm_out,
                       G, N, d.B, k32, hist, st, nblk, sfx, gthi);
    norm = norm_out;
  } else {
    hipLaunchKernelGGL((select_hist_kernel<0, false, SLOTS>), grid, block, 0, s, norm, nullptr, 1, N,
                       d.B, k32, hist, st, nblk, sfx, gthi);
  }
  hipLaunchKernelGGL((select_hist_kernel<1, false, SLOTS>), grid, block, 0, s, norm, nullptr, 1, N, d.B,
                     k32, hist, st, nblk, sfx, gthi);
  hipLaunchKernelGGL((select_hist_kernel<2, false, SLOTS>), grid, block, 0, s, norm, nullptr, 1, N, d.B,
                     k32, hist, st, nblk, sfx, gthi);
  hipLaunchKernelGGL((select_emit_kernel<SLOTS>), grid, block, 0, s, norm, N, k, hist, st, sfx, gthi,
                     nblk, idx, jmap, top_part, G, d.B, block_top);
  return hipGetLastError();
}

hipError_t launch_select(const wcc_desc &d, const float *norm_or_part, int G, float *norm_out,
                         int64_t k, void *ws_base, const WsLayout &L, int32_t *idx, int32_t *jmap,
                         float *top_part, float *block_top, hipStream_t s) {
  const int64_t N = (int64_t)d.H * d.W;
  char *ws = static_cast<char *>(ws_base);
  uint32_t *hist = reinterpret_cast<uint32_t *>(ws + L.hist);
  SelectState *st = reinterpret_cast<SelectState *>(ws + L.state);
  uint16_t *sfx = reinterpret_cast<uint16_t *>(ws + L.block_sfx);
  uint32_t *gthi = reinterpret_cast<uint32_t *>(ws + L.block_gthi);
  const int nblk = L.nblk;
  const uint32_t k32 = (uint32_t)k;
  if (N <= kSmallMaxN) {
    const int slots = (int)((N + 4 * kSmallThreads - 1) / (4 * kSmallThreads));
    if (G >= kCombineGroups && (int64_t)G * N >= kCombineValues) {
      hipLaunchKernelGGL(combine_parts_kernel, dim3((unsigned)((N + 1023) / 1024), d.B), dim3(256), 0, s,
                         norm_or_part, norm_out, G, N, d.B, top_part);
      hipLaunchKernelGGL((select_small_kernel<false>), dim3(d.B), dim3(kSmallThreads), 0, s, norm_out,
                         nullptr, 1, N, d.B, k32, slots, idx, jmap, top_part, block_top);
    } else if (G > 1)
      hipLaunchKernelGGL((select_small_kernel<true>), dim3(d.B), dim3(kSmallThreads), 0, s,
                         norm_or_part, norm_out, G, N, d.B, k32, slots, idx, jmap, top_part, block_top);
    else
      hipLaunchKernelGGL((select_small_kernel<false>), dim3(d.B), dim3(kSmallThreads), 0, s,
                         norm_or_part, nullptr, 1, N, d.B, k32, slots, idx, jmap, top_part, block_top);
    return hipGetLastError();
  }
  switch (L.sel_slots) {
    case 4: return launch_passes<4>(d, norm_or_part, G, norm_out, k, hist, st, sfx, gthi, nblk, idx, jmap, top_part, block_top, s);
    case 2: return launch_passes<2>(d, norm_or_part, G, norm_out, k, hist, st, sfx, gthi, nblk, idx, jmap, top_part, block_top, s);
    default: return launch_passes<1>(d, norm_or_part, G, norm_out, k, hist, st, sfx, gthi, nblk, idx, jmap, top_part, block_top, s);
  }
}

hipError_t launch_jmap_from_idx(const int32_t *idx, int B, int64_t N, int64_t k, int32_t *jmap,
                                hipStream_t s) {
  const int64_t n = (int64_t)B * N;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, jmap, n, -1);
  dim3 grid((unsigned)((k + 255) / 256), B);
  hipLaunchKernelGGL(jmap_scatter_kernel, grid, dim3(256), 0, s, idx, N, k, jmap);
  return hipGetLastError();
}

}  // namespace wcc
