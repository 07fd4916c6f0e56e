// Zero filling and the inverse transform (the decompression step after Eq. wavelet_transform;
// the last loop of Alg. 1), with the skip connection of the inverted residual block.
#include "strip_io.h"

namespace wcc {
namespace {

// ---- synthesis with zero filling ------------------------------------------------------------
// On this chip loads and stores retire through one in-order counter: a load issued after a
// store cannot be waited for without waiting for the store.  A wave that alternates "fetch the
// kept values of channel c, rebuild, store" therefore pays a full store round trip per channel.
// The kernel below issues the fetches of channel c + 1 BEFORE the stores of channel c, with
// the same number of memory instructions on every path (no branch around a load or a store),
// so that waiting for them only needs the stores of channel c - 1 to have retired.
//
// To make that cheap the kept positions of a strip -- the same for every channel, and few --
// are packed once per wave into a list (rank j, cell), slot by slot and lane by lane, held in
// registers, 64 entries a row.  Per channel the wave fetches yc[.., j] for the whole list with
// a few dense loads (neighbouring entries have mostly neighbouring j), drops the values into an
// LDS tile laid out [lane][slot] whose other cells stay zero, and every lane reads its slots
// back from there with 16-byte reads.  Lanes outside the plane take part in the list work; their
// stores carry an offset beyond the plane, which the hardware drops.  Strips that keep more than kInvCap positions, layers with more than 2^20
// kept positions, and d = 4 (whose tile would not fit) take the plain path: ranks in registers,
// one conditional load per slot.
// The channel walk of the staged path with NI dense fetches per channel.  mine[i]: the lane's
// list entries.  PADDED: entries past the end of the list repeat its first entry (they fetch the
// same value and drop it into the same cell), so no load and no LDS write needs a lane mask or
// a branch around it; otherwise padding is kInvNone and is skipped (an empty list).
// dst: the first channel's plane of y (wave-uniform; the next channel's is dst_step elements
// on), off: byte offset of the lane's first row in it, row_bytes: bytes between its rows.
// BUF: rows go through a buffer descriptor of the plane, and lanes outside the plane carry
// off = kRowDropped, row_bytes = 0; waves whose 64 lanes are all inside the plane use plain
// pointers instead (measured 2 % faster on workload 3's inverse).
// RES: the same rows of res (the skip connection's planes) are added to every stored row.
template <int D, int V, int NI, bool RES, class YT, bool PADDED, bool BUF>
__device__ __forceinline__ void inv_staged_walk(const float *__restrict__ plane, int64_t k, int n_ch,
                                                const uint32_t (&mine)[kInvCap / kWave],
                                                uint32_t *tile, const uint32_t *row,
                                                const LanePos<D> &p, YT *dst, uint32_t off,
                                                uint32_t row_bytes, int64_t dst_step, int64_t n,
                                                const YT *res) {
  constexpr int NSP = (slot_count(D, V) + 3) / 4 * 4;  // the lane's slots, whole 16-byte words
  constexpr int R = 1 << D;
  constexpr uint32_t kRank = (1u << kInvRankBits) - 1u;
  float vn[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i)
    vn[i] = plane[(!PADDED && mine[i] == kInvNone) ? 0u : (mine[i] & kRank)];
  auto channel = [&](int c) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
      if (PADDED || mine[i] != kInvNone) tile[mine[i] >> kInvRankBits] = __float_as_uint(vn[i]);
    // the next channel's values travel while this one is built (past the end: the last again)
    const float *nx = plane + (size_t)min(c + 1, n_ch - 1) * k;
#pragma unroll
    for (int i = 0; i < NI; ++i)
      vn[i] = nx[(!PADDED && mine[i] == kInvNone) ? 0u : (mine[i] & kRank)];
    float skip[RES ? R : 1][V];
    if constexpr (RES && BUF) {
      const __amdgpu_buffer_rsrc_t from = plane_rsrc(res, n);
#pragma unroll
      for (int r = 0; r < R; ++r) load_row_buf<V>(from, off + r * row_bytes, skip[r], YT{});
    } else if constexpr (RES) {
      const YT *from = reinterpret_cast<const YT *>(reinterpret_cast<const char *>(res) + off);
#pragma unroll
      for (int r = 0; r < R; ++r) load_row_stream<V>(from + (size_t)r * (row_bytes / sizeof(YT)), skip[r]);
    }
    __builtin_amdgcn_sched_barrier(0);
    wave_lds_fence();
    float out[R][V];
    {
      // the lane's slots come back with NSP / 4 16-byte reads: cells of positions that are not
      // kept hold zero, so there is nothing to test and no branch
      float cells[NSP];
#pragma unroll
      for (int q = 0; q < NSP / 4; ++q) {
        const float4 t = reinterpret_cast<const float4 *>(row)[q];
        cells[4 * q] = t.x; cells[4 * q + 1] = t.y; cells[4 * q + 2] = t.z; cells[4 * q + 3] = t.w;
      }
      const RegStrip<D, V, NSP> src{cells};
      inv_levels<D, V, 1>(out, p, src);
    }
    wave_lds_fence();
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (RES) {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < V; ++e) out[r][e] += skip[r][e];
      res += dst_step;
    }
    if constexpr (BUF) {
      const __amdgpu_buffer_rsrc_t to = plane_rsrc(dst, n);
#pragma unroll
      for (int r = 0; r < R; ++r) store_row_buf<V>(to, off + r * row_bytes, out[r], YT{});
    } else {
      YT *to = reinterpret_cast<YT *>(reinterpret_cast<char *>(dst) + off);
#pragma unroll
      for (int r = 0; r < R; ++r) store_row_stream<V>(to + (size_t)r * (row_bytes / sizeof(YT)), out[r]);
    }
    dst += dst_step;
  };
  // The first channel stands outside the loop: at the loop head the outstanding memory
  // operations are then "fetches, then R stores" on both incoming paths, and the wait for a
  // fetch need not cover the stores.
  channel(0);
  for (int c = 1; c < n_ch; ++c) channel(c);
}

// yc [B, C, k] + jmap [B, N] -> y [B, C, H, W].  grid = (ceil(units/4), G, B), block = 256.
// scratch: unused (kept for the launcher's signature).  RES: y = residual + (the above),
// residual [B, C, H, W] (the skip connection of Eq. (inverted)); it may be y itself.
// YT: float or bf16_t, the storage type of y and of the residual.
template <int D, int V, bool RES, class YT>
__global__ __launch_bounds__(256) void scatter_ihaar_kernel(const float *__restrict__ yc,
                                                            const int32_t *__restrict__ jmap,
                                                            YT *y, Geo g, StripMap m, int C,
                                                            int G, int64_t k, float *scratch,
                                                            const YT *residual) {
  constexpr int R = 1 << D;
  constexpr int NS = slot_count(D, V);
  constexpr bool kStaged = D <= 3;  // the [lane][slot] tiles of four waves fit in LDS
  constexpr int CAP = NS * kWave < kInvCap ? NS * kWave : kInvCap;  // entries a wave can pack
  constexpr int STRIDE = tile_stride((NS + 3) / 4 * 4);  // words between two lanes' slots
  static_assert(NS <= 128, "slot mask is 128 bits wide");
  static_assert(!kStaged || STRIDE * kWave <= (1 << (32 - kInvRankBits)), "cell index fits above the rank");
  __shared__ __attribute__((aligned(16))) uint32_t tiles[kStaged ? 4 : 1][kStaged ? STRIDE * kWave : 1];
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + wv;
  // Samples are taken last to first: the contraction wrote yc first to last, so what is still
  // in the memory-side cache when this kernel starts is the tail, and it is read before the
  // rest of the reads push it out.
  const int grp = blockIdx.y, b = gridDim.z - 1 - blockIdx.z;
  LanePos<D> p;
  int row0, col0;
  const bool active = locate<D, V>(m, g, unit, p, row0, col0);
  // Group grp takes the channels grp, grp + G, grp + 2G, ...: the groups that run side by side
  // then write neighbouring planes of y, a window of G planes that moves through the tensor,
  // instead of G windows a group's width apart (workload 2's inverse 29.6 -> 27.3 us, the
  // block's expand layer 503 -> 478 us).
  const int c0 = grp;
  const int n_ch = c0 >= C ? 0 : (C - c0 + G - 1) / G;
  if (__ballot(active) == 0 || n_ch <= 0) return;  // whole waves leave
  const int64_t kstep = (int64_t)G * k, nstep = (int64_t)G * g.N;

  const int32_t *jm = jmap + (size_t)b * g.N;
  const float *plane = yc + ((size_t)b * C + c0) * k;
  const size_t first = ((size_t)b * C + c0) * g.N + (size_t)row0 * g.W + col0;
  YT *dst = y + first;

  // ranks of this lane's positions (the same for every channel), slot by slot
  InvDirect<D, V> src;
  src.any[0] = src.any[1] = 0;
  int count = 0;  // kept positions of this wave's strip (wave-uniform)
  auto fetch = [&](auto Lc, auto Jc) {
    constexpr int L = decltype(Lc)::value, J = decltype(Jc)::value;
    constexpr int CV = cols_at(V, L);
#pragma unroll
    for (int i = 0; i < rows_at(D, L); ++i)
#pragma unroll
      for (int e = 0; e < CV; ++e) {
        constexpr int base = slot_base(D, V, L, J);
        int j = -1;
        if (active) j = jm[J * p.nl[L] + p.off[L] + i * p.rowlen[L] + e];
        src.jj[base + i * CV + e] = j;
      }
  };
  auto each_level = [&](auto Lc) {
    constexpr int L = decltype(Lc)::value;
    fetch(Lc, std::integral_constant<int, 1>{});
    fetch(Lc, std::integral_constant<int, 2>{});
    fetch(Lc, std::integral_constant<int, 3>{});
    if constexpr (L == D) fetch(Lc, std::integral_constant<int, 0>{});
  };
  each_level(std::integral_constant<int, 1>{});
  if constexpr (D >= 2) each_level(std::integral_constant<int, 2>{});
  if constexpr (D >= 3) each_level(std::integral_constant<int, 3>{});
  if constexpr (D >= 4) each_level(std::integral_constant<int, 4>{});
  // (all map loads are in flight before the first vote waits for one)
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const uint64_t kept = __ballot(src.jj[s] >= 0);
    if (kept != 0) src.any[s >> 6] |= (uint64_t)1 << (s & 63);
    count += __popcll(kept);
  }

  if constexpr (kStaged) {
    if (count <= CAP && k <= ((int64_t)1 << kInvRankBits)) {
      // pack (rank, cell): slot-major, then lane (a band row's kept positions have consecutive
      // j).  The tile serves as scratch for the list before it becomes the staging area.
      uint32_t *tile = tiles[wv];
      int running = 0;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        if ((src.any[s >> 6] >> (s & 63)) & 1) {
          const int j = src.jj[s];
          const uint64_t kept = __ballot(j >= 0);
          const int at = running + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(kept >> 32),
                                       __builtin_amdgcn_mbcnt_lo((uint32_t)kept, 0u));
          if (j >= 0) tile[at] = (uint32_t)j | ((uint32_t)(lane * STRIDE + s) << kInvRankBits);
          running += __popcll(kept);
        }
      }
      wave_lds_fence();
      uint32_t mine[kInvCap / kWave];  // this lane's share of the list: entries lane + 64 i
      const uint32_t pad = count > 0 ? tile[0] : kInvNone;  // (see inv_staged_walk: PADDED)
#pragma unroll
      for (int i = 0; i < kInvCap / kWave; ++i) {
        const int e = lane + 64 * i;
        mine[i] = (i < CAP / kWave && e < count) ? tile[e] : pad;
      }
      wave_lds_fence();
      uint32_t *row = tile + lane * STRIDE;  // this lane's slots
#pragma unroll
      for (int s = 0; s < (NS + 3) / 4 * 4; ++s) row[s] = 0u;
      // the wave's planes (one descriptor per channel) and the lane's place in them
      const size_t plane0 = ((size_t)b * C + c0) * g.N;
      YT *to = y + plane0;
      const YT *res = RES ? residual + plane0 : nullptr;
      const uint32_t off = active ? (uint32_t)(((size_t)row0 * g.W + col0) * sizeof(YT)) : kRowDropped;
      const uint32_t row_bytes = active ? (uint32_t)(g.W * sizeof(YT)) : 0u;
      const int ni = (count + 63) >> 6;
      auto walk = [&](auto buf_c) {
        constexpr bool BUF = decltype(buf_c)::value;
        if (count == 0)  // nothing kept in this strip: rows of zeros (plus the skip connection)
          inv_staged_walk<D, V, 4, RES, YT, false, BUF>(plane, kstep, n_ch, mine, tile, row, p, to, off, row_bytes, nstep, g.N, res);
        else if (ni <= 4)
          inv_staged_walk<D, V, 4, RES, YT, true, BUF>(plane, kstep, n_ch, mine, tile, row, p, to, off, row_bytes, nstep, g.N, res);
        else if (ni <= 8)
          inv_staged_walk<D, V, 8, RES, YT, true, BUF>(plane, kstep, n_ch, mine, tile, row, p, to, off, row_bytes, nstep, g.N, res);
        else
          inv_staged_walk<D, V, 16, RES, YT, true, BUF>(plane, kstep, n_ch, mine, tile, row, p, to, off, row_bytes, nstep, g.N, res);
      };
      if (__ballot(active) == ~0ull) walk(std::false_type{});
      else walk(std::true_type{});
      return;
    }
  }

  // plain path
  if (!active) return;
  src.plane = plane;
  const YT *res = RES ? residual + first : nullptr;
  for (int c = 0; c < n_ch; ++c) {
    float out[R][V];
    inv_levels<D, V, 1>(out, p, src);
    if constexpr (RES) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float skip[V];
        load_row_stream<V>(res + (size_t)r * g.W, skip);
#pragma unroll
        for (int e = 0; e < V; ++e) out[r][e] += skip[e];
      }
      res += nstep;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) store_row_stream<V>(dst + (size_t)r * g.W, out[r]);
    src.plane += kstep;
    dst += nstep;
  }
}

template <int D, int V>
hipError_t inv_launch(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap, void *y,
                      int G, float *scratch, const void *residual, hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = make_map(d, V);
  dim3 grid((m.units + 3) / 4, G, d.B);
#define WCC_INV(RES, YT)                                                                          \
  hipLaunchKernelGGL((scatter_ihaar_kernel<D, V, RES, YT>), grid, dim3(256), 0, s, yc, jmap,      \
                     static_cast<YT *>(y), g, m, d.C_out, G, k, scratch,                          \
                     static_cast<const YT *>(residual))
  if (d.act_dtype == WCC_BF16) { if (residual) WCC_INV(true, bf16_t); else WCC_INV(false, bf16_t); }
  else                         { if (residual) WCC_INV(true, float); else WCC_INV(false, float); }
#undef WCC_INV
  return hipGetLastError();
}

}  // namespace

hipError_t inv_dispatch(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap, void *y,
                        int G, float *scratch, const void *residual, hipStream_t s) {
  const bool v4 = d.W % 4 == 0;
  switch (d.levels) {
    case 1: return v4 ? inv_launch<1, 4>(d, k, yc, jmap, y, G, scratch, residual, s)
                      : inv_launch<1, 2>(d, k, yc, jmap, y, G, scratch, residual, s);
    case 2: return inv_launch<2, 4>(d, k, yc, jmap, y, G, scratch, residual, s);
    case 3: return inv_launch<3, 4>(d, k, yc, jmap, y, G, scratch, residual, s);
    case 4: return inv_launch<4, 4>(d, k, yc, jmap, y, G, scratch, residual, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_scatter_ihaar(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap,
                                void *y, float *scratch, const void *residual, hipStream_t s) {
  return inv_dispatch(d, k, yc, jmap, y, groups_for(d, d.C_out, 4096, 4), scratch, residual, s);
}

}  // namespace wcc
