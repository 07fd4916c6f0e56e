// Joint shrinkage (Alg. 1: "indices of the top ceil(gamma n_w n_h) vectors by norm"):
// per sample, the k largest of N non-negative fp32 norms, ties toward the lower position,
// emitted in ascending position order.
//
// Design.  Non-negative floats order like their bit patterns, so the k-th largest norm is
// found exactly by a most-significant-digit radix select on uint32 keys: three histogram
// passes (11 + 11 + 10 bits) spread over many workgroups per sample, integer atomics only.
// The workgroup that finishes a pass last (counted with a device-scope atomic after a
// fence) turns the histogram into the digit to descend into; nobody spins on anybody.
// With the threshold key T and the number r of keys equal to T still to take, a counting
// pass and an ordered compaction write idx: a position is kept if key > T, or key == T and
// fewer than r equal keys precede it.  Ordering comes from prefix sums, never from the
// arrival order of atomics, so the result is the same on every run.
#include "wcc_internal.h"

namespace wcc {
namespace {

constexpr int kThreads = 256;
constexpr int kPerThread = kSelectChunk / kThreads;  // 16 keys per thread

__device__ __forceinline__ uint32_t digit_of(uint32_t key, int pass) {
  return pass == 0 ? key >> 21 : pass == 1 ? (key >> 10) & 0x7FFu : key & 0x3FFu;
}
// keys whose bits above the current digit equal `prefix`
__device__ __forceinline__ bool matches(uint32_t key, uint32_t prefix, int pass) {
  return pass == 0 ? true : pass == 1 ? (key >> 21) == (prefix >> 21) : (key >> 10) == (prefix >> 10);
}

// zero histograms and per-sample state; state.remain = k
__global__ __launch_bounds__(kThreads) void select_init_kernel(uint32_t *hist, SelectState *st,
                                                               int B, uint32_t k) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B * 3 * kRadixBins) hist[i] = 0;
  if (i < B) {
    SelectState s;
    s.prefix = 0; s.remain = k;
    s.done[0] = s.done[1] = s.done[2] = 0;
    s.pad[0] = s.pad[1] = s.pad[2] = 0;
    st[i] = s;
  }
}

// One histogram pass.  grid = (nblk, B).
template <int PASS>
__global__ __launch_bounds__(kThreads) void select_hist_kernel(const float *__restrict__ norm,
                                                               int64_t N, uint32_t *hist,
                                                               SelectState *st, int nblk) {
  __shared__ uint32_t lh[kRadixBins];
  __shared__ uint32_t scan[kThreads];
  __shared__ int is_last;
  const int b = blockIdx.y, t = threadIdx.x;
  const uint32_t *keys = reinterpret_cast<const uint32_t *>(norm) + (size_t)b * N;
  uint32_t *gh = hist + ((size_t)b * 3 + PASS) * kRadixBins;
  SelectState *s = st + b;
  constexpr int bins = PASS == 2 ? 1024 : kRadixBins;

  for (int i = t; i < bins; i += kThreads) lh[i] = 0;
  __syncthreads();
  const uint32_t prefix = PASS == 0 ? 0u : s->prefix;
  const int64_t base = (int64_t)blockIdx.x * kSelectChunk;
#pragma unroll 4
  for (int r = 0; r < kPerThread; ++r) {
    const int64_t q = base + r * kThreads + t;
    if (q < N) {
      const uint32_t key = keys[q];
      if (matches(key, prefix, PASS)) atomicAdd(&lh[digit_of(key, PASS)], 1u);
    }
  }
  __syncthreads();
  for (int i = t; i < bins; i += kThreads) {
    const uint32_t v = lh[i];
    if (v) atomicAdd(&gh[i], v);
  }
  // last workgroup of this sample to finish picks the digit
  __threadfence();
  __syncthreads();
  if (t == 0) {
    const uint32_t prev = atomicAdd(&s->done[PASS], 1u);
    is_last = (prev == (uint32_t)nblk - 1);
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();

  // descending cumulative count: find digit D with count(> D) < remain <= count(>= D)
  constexpr int per = bins / kThreads;  // 8 (or 4) consecutive digits per thread, from the top
  const uint32_t remain = s->remain;
  uint32_t cnt[per], sum = 0;
#pragma unroll
  for (int i = 0; i < per; ++i) {
    cnt[i] = __hip_atomic_load(&gh[bins - 1 - (t * per + i)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sum += cnt[i];
  }
  scan[t] = sum;
  __syncthreads();
  // exclusive prefix over threads (threads ordered from the top digit down)
  for (int off = 1; off < kThreads; off <<= 1) {
    uint32_t v = (t >= off) ? scan[t - off] : 0;
    __syncthreads();
    scan[t] += v;
    __syncthreads();
  }
  uint32_t above = scan[t] - sum;  // keys in digits above this thread's digits
#pragma unroll
  for (int i = 0; i < per; ++i) {
    if (above < remain && remain <= above + cnt[i]) {
      const uint32_t digit = bins - 1 - (t * per + i);
      const uint32_t shifted = PASS == 0 ? digit << 21 : PASS == 1 ? digit << 10 : digit;
      s->prefix = prefix | shifted;
      s->remain = remain - above;
    }
    above += cnt[i];
  }
}

// block-wide exclusive scan of a packed pair (hi16: gt, lo16: eq); returns the block total too
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot,
                                                         uint32_t &total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t n = __shfl_up(inc, off, 64);
    if (lane >= off) inc += n;
  }
  if (lane == 63) wave_tot[wv] = inc;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kThreads / 64; ++i) {
    const uint32_t w = wave_tot[i];
    if (i < wv) before += w;
    tot += w;
  }
  total = tot;
  return before + inc - v;
}

// per-workgroup counts of keys above / equal to the threshold.  grid = (nblk, B)
__global__ __launch_bounds__(kThreads) void select_count_kernel(const float *__restrict__ norm,
                                                                int64_t N, const SelectState *st,
                                                                uint2 *blockcnt, int nblk) {
  __shared__ uint32_t wave_tot[kThreads / 64];
  const int b = blockIdx.y, t = threadIdx.x;
  const uint32_t *keys = reinterpret_cast<const uint32_t *>(norm) + (size_t)b * N;
  const uint32_t T = st[b].prefix;
  const int64_t base = (int64_t)blockIdx.x * kSelectChunk + (int64_t)t * kPerThread;
  uint32_t packed = 0;
  if (base < N) {
#pragma unroll
    for (int r = 0; r < kPerThread; r += 4) {
      if (base + r < N) {  // N is a multiple of 4
        const uint4 k4 = *reinterpret_cast<const uint4 *>(keys + base + r);
        packed += ((k4.x > T) << 16) + (k4.x == T);
        packed += ((k4.y > T) << 16) + (k4.y == T);
        packed += ((k4.z > T) << 16) + (k4.z == T);
        packed += ((k4.w > T) << 16) + (k4.w == T);
      }
    }
  }
  uint32_t total;
  (void)block_exclusive_scan(packed, wave_tot, total);
  if (t == 0) blockcnt[(size_t)b * nblk + blockIdx.x] = make_uint2(total >> 16, total & 0xFFFFu);
}

// ordered compaction.  grid = (nblk, B).  jmap (nullable) gets the rank of every kept
// position and -1 for every dropped one.
__global__ __launch_bounds__(kThreads) void select_emit_kernel(const float *__restrict__ norm,
                                                               int64_t N, int64_t k,
                                                               const SelectState *st,
                                                               const uint2 *blockcnt, int nblk,
                                                               int32_t *__restrict__ idx,
                                                               int32_t *__restrict__ jmap) {
  __shared__ uint32_t wave_tot[kThreads / 64];
  __shared__ uint32_t red[2][kThreads / 64];
  const int b = blockIdx.y, t = threadIdx.x;
  const uint32_t *keys = reinterpret_cast<const uint32_t *>(norm) + (size_t)b * N;
  const uint32_t T = st[b].prefix, r_take = st[b].remain;

  // keys above / equal to T in the workgroups before this one
  uint32_t gt0 = 0, eq0 = 0;
  for (int i = t; i < (int)blockIdx.x; i += kThreads) {
    const uint2 c = blockcnt[(size_t)b * nblk + i];
    gt0 += c.x; eq0 += c.y;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    gt0 += __shfl_down(gt0, off, 64);
    eq0 += __shfl_down(eq0, off, 64);
  }
  if ((t & 63) == 0) { red[0][t >> 6] = gt0; red[1][t >> 6] = eq0; }
  __syncthreads();
  gt0 = red[0][0] + red[0][1] + red[0][2] + red[0][3];
  eq0 = red[1][0] + red[1][1] + red[1][2] + red[1][3];

  const int64_t base = (int64_t)blockIdx.x * kSelectChunk + (int64_t)t * kPerThread;
  uint32_t key[kPerThread];
  uint32_t packed = 0;
#pragma unroll
  for (int r = 0; r < kPerThread; r += 4) {
    uint4 k4 = make_uint4(0, 0, 0, 0);
    if (base + r < N) k4 = *reinterpret_cast<const uint4 *>(keys + base + r);
    key[r] = k4.x; key[r + 1] = k4.y; key[r + 2] = k4.z; key[r + 3] = k4.w;
  }
#pragma unroll
  for (int r = 0; r < kPerThread; ++r)
    if (base + r < N) packed += ((key[r] > T) << 16) + (key[r] == T);
  uint32_t total;
  const uint32_t ex = block_exclusive_scan(packed, wave_tot, total);
  uint32_t gt = gt0 + (ex >> 16), eq = eq0 + (ex & 0xFFFFu);

  int32_t *out = idx + (size_t)b * k;
  int32_t *jm = jmap ? jmap + (size_t)b * N : nullptr;
#pragma unroll
  for (int r = 0; r < kPerThread; ++r) {
    const int64_t q = base + r;
    if (q >= N) break;
    const bool is_gt = key[r] > T, is_eq = key[r] == T;
    const bool keep = is_gt || (is_eq && eq < r_take);
    const uint32_t j = gt + min(eq, r_take);
    if (keep) out[j] = (int32_t)q;
    if (jm) jm[q] = keep ? (int32_t)j : -1;
    gt += is_gt; eq += is_eq;
  }
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

}  // namespace

hipError_t launch_select(const wcc_desc &d, const float *norm, int64_t k, void *ws_base,
                         const WsLayout &L, int32_t *idx, int32_t *jmap, hipStream_t s) {
  const int64_t N = (int64_t)d.H * d.W;
  char *ws = static_cast<char *>(ws_base);
  uint32_t *hist = reinterpret_cast<uint32_t *>(ws + L.hist);
  SelectState *st = reinterpret_cast<SelectState *>(ws + L.state);
  uint2 *blockcnt = reinterpret_cast<uint2 *>(ws + L.blockcnt);
  const int nblk = L.nblk;
  const int init_n = d.B * 3 * kRadixBins;
  hipLaunchKernelGGL(select_init_kernel, dim3((init_n + kThreads - 1) / kThreads), dim3(kThreads),
                     0, s, hist, st, d.B, (uint32_t)k);
  dim3 grid(nblk, d.B);
  hipLaunchKernelGGL(select_hist_kernel<0>, grid, dim3(kThreads), 0, s, norm, N, hist, st, nblk);
  hipLaunchKernelGGL(select_hist_kernel<1>, grid, dim3(kThreads), 0, s, norm, N, hist, st, nblk);
  hipLaunchKernelGGL(select_hist_kernel<2>, grid, dim3(kThreads), 0, s, norm, N, hist, st, nblk);
  hipLaunchKernelGGL(select_count_kernel, grid, dim3(kThreads), 0, s, norm, N, st, blockcnt, nblk);
  hipLaunchKernelGGL(select_emit_kernel, grid, dim3(kThreads), 0, s, norm, N, k, st, blockcnt, nblk,
                     idx, jmap);
  return hipGetLastError();
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
