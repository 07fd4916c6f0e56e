// Compressed-domain chaining of the inverted residual block (appendix "Inference times",
// paragraph on memory bandwidth and traffic: Haar transform, depthwise convolution and
// gather / scatter applied separately per channel and in parts, with small intermediates, the
// full result kept only in compressed form).
//
// The project layer's input is K_dw t1 with t1 = iHWT(T^T Y_wt) the expand layer's output.  The
// two transform passes of the project layer (channel norms; kept coefficients) take t1 from
// where it already is in compressed form -- the expand layer's Y_wt [B, C, k] and its rank map
// -- instead of from a feature map in memory: per channel a wave rebuilds the 2^d rows of its
// strip and the one row above and below it (inverse transform of the kept values, everything
// else zero), convolves them with the channel's 3x3 kernel and transforms the result again, all
// in registers and LDS.  The expanded feature map, the largest tensor of the block, is neither
// written nor read; the passes read k/N of it, twice.  This is also the mirror fusion "inverse
// transform followed by the depthwise convolution".
//
// The arithmetic is that of the kernels it replaces, operation by operation (synthesis
// butterflies of haar_inv.hip, multiply-adds in the order of depthwise.hip, analysis of strip.h),
// so the values that enter the norms and the quantiser are the same bits.
//
// A row of the plane wider than one wave row (256 columns) is shared by the 2 or 4 waves of a
// workgroup, one 256-column segment each: per channel every wave leaves the first and last
// column of its rebuilt rows in LDS, the workgroup meets at a barrier, and the end lanes take the
// convolution's outside column from the neighbouring segment there.
//
// Limits (the caller falls back to the materialised route otherwise): W % 4 == 0, d <= 3, and
// W <= 256 or a row made of exactly 2 or 4 wave rows (256 < W <= 512, 768 < W <= 1024).
#include "strip_io.h"

namespace wcc {
namespace {

constexpr int V4 = 4;

// ---- slots of ONE row of a strip (the halo rows) -------------------------------------------------
// To rebuild a single image row only the band row that contains it is needed at every level.
__host__ __device__ constexpr int hslot_base(int D, int V, int l, int j) {
  int s = 0;
  for (int m = 1; m < l; ++m) s += 3 * cols_at(V, m);
  return s + (l == D ? j : j - 1) * cols_at(V, l);
}
__host__ __device__ constexpr int hslot_count(int D, int V) {
  return hslot_base(D, V, D, 3) + cols_at(V, D);
}

// (the [lane][slot] tile layout and RegStrip, the source that reads a lane's slots back from
// registers, are in strip_io.h: the inverse transform uses them too)
template <int D, int V, int N>
struct RegRow {
  const float (&c)[N];
  int first;  // the halo row's first slot
  template <int L, int J>
  __device__ __forceinline__ void get(float (&v)[cols_at(V, L)]) const {
    constexpr int CV = cols_at(V, L);
    constexpr int base = hslot_base(D, V, L, J);
#pragma unroll
    for (int e = 0; e < CV; ++e) v[e] = c[first + base + e];
  }
};

// One image row of a strip: its last one (BOTTOM) or its first one.  The same expressions as
// inv_levels evaluates for that row.
template <int D, int V, int L, bool BOTTOM, class Source>
__device__ __forceinline__ void inv_row(float (&out)[cols_at(V, L - 1)], const LanePos<D> &p,
                                        const Source &src) {
  constexpr int VI = cols_at(V, L - 1), V2 = cols_at(V, L);
  constexpr int SI = span_at(V, L - 1);
  float ll[V2];
  if constexpr (L < D) inv_row<D, V, L + 1, BOTTOM>(ll, p, src);
  else src.template get<L, 0>(ll);
  float y2[V2], y3[V2], y4[V2];
  src.template get<L, 1>(y2);
  src.template get<L, 2>(y3);
  src.template get<L, 3>(y4);
#pragma unroll
  for (int e = 0; e < V2; ++e) {
    const float s1 = ll[e] + y3[e], s2 = ll[e] - y3[e];
    const float d1 = y2[e] + y4[e], d2 = y2[e] - y4[e];
    const float l = BOTTOM ? 0.5f * (s2 + d2) : 0.5f * (s1 + d1);
    const float r = BOTTOM ? 0.5f * (s2 - d2) : 0.5f * (s1 - d1);
    if constexpr (VI >= 2) {
      out[2 * e] = l;
      out[2 * e + 1] = r;
    } else {
      out[0] = ((p.lc & SI) == 0) ? l : r;
    }
  }
}

// ---- the channel walk ----------------------------------------------------------------------------
constexpr int kChainCap = 2048;  // packed entries per wave (32 a lane)

// What a wave knows about the producer layer's kept positions around its strip.
template <int D>
struct ChainGeo {
  static constexpr int NS = slot_count(D, V4), HS = hslot_count(D, V4), NT = NS + 2 * HS;
  static constexpr int STRIDE = tile_stride(NT);  // words between two lanes' slots in the tile
  uint64_t any;        // wave-uniform: bit s set if some lane keeps slot s (NT <= 64)
  int count;           // kept entries of the wave (wave-uniform)
  bool packed;         // the tile holds the wave's packed list (rank | cell << kInvRankBits)
  int jj[NT];          // rank in the producer's list of the lane's slot, or -1 (used if !packed)
};

// Calls f(slot, position in the producer's rank map, exists) for the lane's NT slots: the strip's
// own NS slots, then the HS slots of the band rows that hold the image row above the strip,
// then those of the row below.
template <int D, class F>
__device__ __forceinline__ void chain_slots(const LanePos<D> &p, bool active, bool up_in, bool dn_in,
                                            F &&f) {
  constexpr int NS = ChainGeo<D>::NS, HS = ChainGeo<D>::HS;
  auto band_rows = [&](auto Lc, auto Jc) {
    constexpr int L = decltype(Lc)::value, J = decltype(Jc)::value;
    constexpr int CV = cols_at(V4, L);
    const int band = J * p.nl[L] + p.off[L];
#pragma unroll
    for (int i = 0; i < rows_at(D, L); ++i)
#pragma unroll
      for (int e = 0; e < CV; ++e) f(slot_base(D, V4, L, J) + i * CV + e, band + i * p.rowlen[L] + e, active);
#pragma unroll
    for (int e = 0; e < CV; ++e) {
      f(NS + hslot_base(D, V4, L, J) + e, band - p.rowlen[L] + e, active && up_in);
      f(NS + HS + hslot_base(D, V4, L, J) + e, band + rows_at(D, L) * p.rowlen[L] + e, active && dn_in);
    }
  };
  auto each_level = [&](auto Lc) {
    constexpr int L = decltype(Lc)::value;
    band_rows(Lc, std::integral_constant<int, 1>{});
    band_rows(Lc, std::integral_constant<int, 2>{});
    band_rows(Lc, std::integral_constant<int, 3>{});
    if constexpr (L == D) band_rows(Lc, std::integral_constant<int, 0>{});
  };
  each_level(std::integral_constant<int, 1>{});
  if constexpr (D >= 2) each_level(std::integral_constant<int, 2>{});
  if constexpr (D >= 3) each_level(std::integral_constant<int, 3>{});
}

// Looks up the lane's slots in the producer's rank map jm1 (one sample) and, if the wave keeps
// at most kChainCap of them (and the ranks fit their bit field), packs (rank, cell) into `tile`:
// slot-major, then lane.
template <int D>
__device__ __forceinline__ ChainGeo<D> chain_setup(const int32_t *__restrict__ jm1, int64_t k1,
                                                   const LanePos<D> &p, bool active, bool up_in,
                                                   bool dn_in, uint32_t *tile) {
  constexpr int NT = ChainGeo<D>::NT;
  static_assert(NT <= 64, "one 64-bit slot mask");
  constexpr int STRIDE = ChainGeo<D>::STRIDE;
  static_assert(STRIDE * kWave <= (1 << (32 - kInvRankBits)), "cell index fits above the rank");
  static_assert(NT % 4 == 0 && STRIDE % 4 == 0, "16-byte reads of a lane's slots");
  const int lane = threadIdx.x & (kWave - 1);
  ChainGeo<D> cg;
  int (&jj)[NT] = cg.jj;
  chain_slots<D>(p, active, up_in, dn_in, [&](int s, int pos, bool exists) {
    int j = -1;
    if (exists) j = jm1[pos];
    jj[s] = j;
  });
  cg.any = 0;
  cg.count = 0;
#pragma unroll
  for (int s = 0; s < NT; ++s) {
    const uint64_t kept = __ballot(jj[s] >= 0);
    if (kept != 0) cg.any |= (uint64_t)1 << s;
    cg.count += __popcll(kept);
  }
  cg.packed = cg.count <= kChainCap && k1 <= ((int64_t)1 << kInvRankBits);
  if (cg.packed) {
    int running = 0;
#pragma unroll
    for (int s = 0; s < NT; ++s) {
      if ((cg.any >> s) & 1) {
        const int j = jj[s];
        const uint64_t kept = __ballot(j >= 0);
        const int at = running + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(kept >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)kept, 0u));
        if (j >= 0) tile[at] = (uint32_t)j | ((uint32_t)(lane * STRIDE + s) << kInvRankBits);
        running += __popcll(kept);
      }
    }
    wave_lds_fence();
  }
  return cg;
}

// Walks n_ch channels of the producer's compressed output yc1 (first channel at `plane`, channel
// stride k1): per channel the kept values around the strip go into the wave's LDS
// tile (laid out [lane][slot]; its other cells stay zero), the strip's 2^d rows and the rows above and below are
// rebuilt from it, convolved with the channel's 3x3 kernel (wdw: first channel's, 9 floats a
// channel) and transformed into `sink`; after(sink) runs once per channel.
// Waves whose list is packed fetch it with dense loads, one or two channels ahead; the others
// (strips that keep more than kChainCap positions) load slot by slot from the ranks they hold in
// registers, a channel's loads in flight together.
// NI_FIXED > 0: the packed list is walked with that many rows a wave (the caller has checked that
// it fits); 0: the shortest of 4, 8, 16, 32 rows that holds it.
// SEGS > 1: the plane's row is shared by the SEGS waves of the workgroup (this one holds segment
// `seg`); xchg is the workgroup's exchange buffer (ChainXchg<D, SEGS>::kWords floats).  Every wave
// of the workgroup then runs compute() once per channel, whatever path it takes: one barrier each.
template <int D, int SEGS, int NI_FIXED = 0, class Sink, class After>
__device__ __forceinline__ void chain_walk(const float *__restrict__ plane, int64_t k1, int n_ch,
                                           const float *__restrict__ wdw, const ChainGeo<D> &cg,
                                           uint32_t *tile, const LanePos<D> &p, bool first_lane,
                                           bool last_lane, float *xchg, int seg, Sink &sink,
                                           After &&after) {
  constexpr int R = 1 << D, RR = R + 2, V = V4;
  int parity = 0;  // which half of the exchange buffer this channel uses
  constexpr int NS = ChainGeo<D>::NS, HS = ChainGeo<D>::HS, NT = ChainGeo<D>::NT;
  constexpr int STRIDE = ChainGeo<D>::STRIDE;
  const int lane = threadIdx.x & (kWave - 1);
  uint32_t *mine_row = tile + lane * STRIDE;  // this lane's slots

  // the tile holds a channel's kept values: rebuild, convolve with kw[0..8], transform
  auto compute = [&](const float *kw) {
    float k[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) k[t] = kw[t];
    wave_lds_fence();
    float six[RR][V + 2];
    {
      float cells[NT];
#pragma unroll
      for (int q = 0; q < NT / 4; ++q) {
        const float4 t = reinterpret_cast<const float4 *>(mine_row)[q];
        cells[4 * q] = t.x; cells[4 * q + 1] = t.y; cells[4 * q + 2] = t.z; cells[4 * q + 3] = t.w;
      }
      const RegStrip<D, V, NT> own{cells};
      const RegRow<D, V, NT> up{cells, NS}, dn{cells, NS + HS};
      float mid[R][V];
      inv_levels<D, V, 1>(mid, p, own);
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < V; ++e) six[r + 1][e + 1] = mid[r][e];
      float edge[V];
      inv_row<D, V, 1, true>(edge, p, up);
#pragma unroll
      for (int e = 0; e < V; ++e) six[0][e + 1] = edge[e];
      inv_row<D, V, 1, false>(edge, p, dn);
#pragma unroll
      for (int e = 0; e < V; ++e) six[RR - 1][e + 1] = edge[e];
    }
    wave_lds_fence();
    // the column beyond a wave row's end: the plane's zero border, or (SEGS > 1) the neighbouring
    // segment's boundary column.  Two buffers alternate: a wave can be one barrier ahead of
    // another, never two, so the buffer it writes is not the one a slower wave still reads.
    float beyond[RR];
#pragma unroll
    for (int i = 0; i < RR; ++i) beyond[i] = 0.f;
    // (a last segment of a single lane: that lane is first and last at once; `beyond` then holds
    // the column to its left, and to its right lies the plane's border)
    bool left_only = false;
    if constexpr (SEGS > 1) {
      float *ex = xchg + parity * (SEGS * 2 * RR);
      parity ^= 1;
      // (the lane number is computed afresh here, by instructions the compiler may not move out
      // of the loop: kept across the loop it is spilled, and the reload of a spilled register
      // waits for every load in flight, the prefetched channels included)
      int ln;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
      const bool at0 = ln == 0, at63 = ln == kWave - 1;
      if (at0 || at63) {
        float *out = ex + (seg * 2 + (at0 ? 0 : 1)) * RR;
#pragma unroll
        for (int i = 0; i < RR; ++i) out[i] = at0 ? six[i][1] : six[i][V];
      }
      workgroup_lds_barrier();  // (the next channels' values keep travelling)
      if ((at0 && seg > 0) || (at63 && seg < SEGS - 1)) {
        const float *in = ex + (at0 ? (seg - 1) * 2 + 1 : (seg + 1) * 2) * RR;
#pragma unroll
        for (int i = 0; i < RR; ++i) beyond[i] = in[i];
      }
      left_only = at0;
    }
#pragma unroll
    for (int i = 0; i < RR; ++i) {
      float l = __shfl_up(six[i][V], 1, kWave), r = __shfl_down(six[i][1], 1, kWave);
      if (first_lane) l = beyond[i];
      if (last_lane) r = left_only ? 0.f : beyond[i];
      six[i][0] = l;
      six[i][V + 1] = r;
    }
    float t1[R][V];
#pragma unroll
    for (int o = 0; o < R; ++o) {
#pragma unroll
      for (int e = 0; e < V; ++e) t1[o][e] = 0.f;
#pragma unroll
      for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
          for (int e = 0; e < V; ++e) t1[o][e] = fmaf(k[i * 3 + j], six[o + i][e + j], t1[o][e]);
    }
    fwd_levels<D, V, 1>(t1, p, sink);
    after(sink);
  };

  if (cg.packed) {
    auto run = [&](auto ni_c) {
      constexpr int NI = decltype(ni_c)::value;
      // Channels of values in flight ahead of the one being worked on: two for short lists, one
      // for longer ones (registers; the 32-row walk spills some of them, which still costs far
      // less than waiting for every channel's values where they are needed).
      constexpr int DEPTH = NI <= 8 ? 2 : 1;
      constexpr uint32_t kRank = (1u << kInvRankBits) - 1u;
      // this lane's share of the list: entries lane + 64 i.  Past the end of the list an entry
      // repeats the list's first one: it fetches the same value and drops it into the same cell,
      // so no load and no LDS write needs a lane mask or a branch.
      uint32_t mine[NI];
      const uint32_t first = tile[0];
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int e = lane + kWave * i;
        mine[i] = e < cg.count ? tile[e] : first;
      }
      wave_lds_fence();
#pragma unroll
      for (int s = 0; s < NT; ++s) mine_row[s] = 0u;
      auto fetch = [&](float (&dst)[NI], int ch) {  // (past the last channel: the last again)
        const float *nx = plane + (size_t)min(ch, n_ch - 1) * k1;
#pragma unroll
        for (int i = 0; i < NI; ++i) dst[i] = nx[mine[i] & kRank];
      };
      auto drop = [&](const float (&src)[NI]) {
#pragma unroll
        for (int i = 0; i < NI; ++i) tile[mine[i] >> kInvRankBits] = __float_as_uint(src[i]);
      };
      if constexpr (DEPTH == 0) {
        for (int c = 0; c < n_ch; ++c) {
          float v[NI];
          fetch(v, c);
          drop(v);
          compute(wdw + (size_t)c * 9);
        }
      } else {
        float vn[DEPTH][NI];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) fetch(vn[u], u);
        int c = 0;
        for (; c + DEPTH <= n_ch; c += DEPTH) {
#pragma unroll
          for (int u = 0; u < DEPTH; ++u) {
            drop(vn[u]);
            fetch(vn[u], c + u + DEPTH);  // travels while the channels in between are worked on
            __builtin_amdgcn_sched_barrier(0);
            compute(wdw + (size_t)(c + u) * 9);
          }
        }
#pragma unroll
        for (int u = 0; u < DEPTH - 1; ++u) {
          if (c + u < n_ch) {
            drop(vn[u]);
            compute(wdw + (size_t)(c + u) * 9);
          }
        }
      }
    };
    if (cg.count == 0) {  // nothing kept around this strip: every channel is zero
#pragma unroll
      for (int s = 0; s < NT; ++s) mine_row[s] = 0u;
      for (int c = 0; c < n_ch; ++c) compute(wdw + (size_t)c * 9);
      return;
    }
    if constexpr (NI_FIXED > 0) {
      run(std::integral_constant<int, NI_FIXED>{});
    } else {
      const int ni = (cg.count + kWave - 1) >> 6;
      if (ni <= 4) run(std::integral_constant<int, 4>{});
      else if (ni <= 8) run(std::integral_constant<int, 8>{});
      else if (ni <= 16) run(std::integral_constant<int, 16>{});
      else run(std::integral_constant<int, 32>{});
    }
    return;
  }

  // plain path: one load per slot that some lane keeps, all of a channel's loads in flight together
#pragma unroll
  for (int s = 0; s < NT; ++s) mine_row[s] = 0u;
  for (int c = 0; c < n_ch; ++c) {
    const float *pc = plane + (size_t)c * k1;
    float v[NT];
#pragma unroll
    for (int s = 0; s < NT; ++s) v[s] = pc[max(cg.jj[s], 0)];
#pragma unroll
    for (int s = 0; s < NT; ++s) mine_row[s] = cg.jj[s] >= 0 ? __float_as_uint(v[s]) : 0u;
    compute(wdw + (size_t)c * 9);
  }
}

// Sink of the keep pass for a strip that keeps few of its positions (the counterpart of
// KeepStagedSink for the [lane][slot] tile): every lane drops its coefficients into its own
// slots of the tile -- free once the channel's rows have been rebuilt from it --, the wave picks
// the values of the strip's packed list of kept positions from there and stores NI dense rows
// (only those are quantised), and the lane's own slots are cleared again for the next channel.
template <int D, bool Q8, int NI>
struct ChainStagedSink {
  using Out = std::conditional_t<Q8, int8_t, float>;
  static constexpr uint32_t kDropped = 0xFFFFFFFFu;
  static constexpr int NS = slot_count(D, V4);
  __amdgpu_buffer_rsrc_t xc_c;  // xc[b, c, :]
  uint32_t *tile;               // the wave's tile
  uint32_t *row;                // this lane's slots in it
  uint32_t cell[NI];            // tile index of the entry's position
  uint32_t at[NI];              // byte offset of the entry's rank, or kDropped (list padding)
  float vmax;
  Quant quant;
  __device__ __forceinline__ explicit ChainStagedSink(float alpha) : quant(alpha) {}
  __device__ __forceinline__ void aim(Out *plane, int64_t k) {
    xc_c = __builtin_amdgcn_make_buffer_rsrc(plane, 0, (int)(uint32_t)(k * (int64_t)sizeof(Out)),
                                             0x00020000 /* raw dwords, no swizzle */);
  }
  template <int L, int J>
  __device__ __forceinline__ void put_row(const LanePos<D> &p, int i, const float (&v)[cols_at(V4, L)],
                                          bool owner) {
    constexpr int CV = cols_at(V4, L);
    constexpr int base = slot_base(D, V4, L, J);
    (void)p;
    (void)owner;  // (a value a lane does not own is in no list)
#pragma unroll
    for (int e = 0; e < CV; ++e) row[base + i * CV + e] = __float_as_uint(v[e]);
  }
  // once per channel, after the last level
  __device__ __forceinline__ void flush() {
    wave_lds_fence();
    if constexpr (Q8) {
      // which division the quantiser takes is the same for every value of the layer: chosen
      // once per channel here, not value by value (three branches a value otherwise)
      float v[NI];
#pragma unroll
      for (int i = 0; i < NI; ++i) v[i] = __uint_as_float(tile[cell[i]]);
      auto store_codes = [&](auto fast_c) {
        constexpr bool FAST = decltype(fast_c)::value;
#pragma unroll
        for (int i = 0; i < NI; ++i)
          __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(int8_t)(int)quant.template level_as<FAST>(v[i]),
                                               xc_c, at[i], 0, 0);
      };
      if (quant.fast) store_codes(std::true_type{});
      else store_codes(std::false_type{});
    } else {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const float v = __uint_as_float(tile[cell[i]]);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), xc_c, at[i], 0, 0);
        vmax = fmaxf(vmax, at[i] != kDropped ? fabsf(v) : 0.f);
      }
    }
    wave_lds_fence();
    // the strip's own slots go back to zero (the slots that round NS up to a multiple of four
    // belong to the row above: zero as well until the next channel's values are dropped in)
#pragma unroll
    for (int q = 0; q < (NS + 3) / 4; ++q) reinterpret_cast<uint4 *>(row)[q] = make_uint4(0u, 0u, 0u, 0u);
    wave_lds_fence();
  }
};

// Waves per workgroup: two (independent of each other when a wave row holds a whole row of the
// plane), so that a workgroup's tiles stay small enough for several workgroups to share a
// compute unit's LDS; with SEGS segments a row, the SEGS waves that share it.
constexpr int kChainWaves = 2;
__host__ __device__ constexpr int chain_waves(int segs) { return segs > 1 ? segs : kChainWaves; }

// the boundary columns of the segments' rebuilt rows: [2 buffers][segment][first | last column][row]
template <int D, int SEGS>
struct ChainXchg {
  static constexpr int kWords = SEGS > 1 ? 2 * SEGS * 2 * ((1 << D) + 2) : 1;
};

// LDS of a workgroup: its waves' [lane][slot] tiles
template <int D>
struct ChainTiles {
  static constexpr int kWords = ChainGeo<D>::STRIDE * kWave;
};

// ---- first pass: channel norms of HWT(K_dw t1) ------------------------------------------------------
// grid = (ceil(units/waves), G, B), block = waves = chain_waves(SEGS) waves.  yc1 [B, C, k1], jmap1 [B, N]: the producer layer's
// compressed output and rank map; wdw [C, 3, 3].  Writes the partial norms (and the partial
// maxima of |coefficient|, nullable) of channel group grp to norm_part / max_part [G, B, N].
template <int D, bool SQ, int SEGS>
__global__ __launch_bounds__(chain_waves(SEGS) * kWave, 4 / chain_waves(SEGS)) void chain_norm_kernel(const float *__restrict__ yc1,
                                                         const int32_t *__restrict__ jmap1,
                                                         int64_t k1, const float *__restrict__ wdw,
                                                         float *__restrict__ norm_part,
                                                         float *__restrict__ max_part, Geo g,
                                                         StripMap m, int C, int Cg, int B,
                                                         SelectPrep prep) {
  constexpr int NS = slot_count(D, V4), WAVES = chain_waves(SEGS);
  __shared__ __attribute__((aligned(16))) uint32_t tiles[WAVES][ChainTiles<D>::kWords];
  __shared__ float xchg[ChainXchg<D, SEGS>::kWords];
  const int wv = threadIdx.x >> 6;
  const int unit = blockIdx.x * WAVES + wv;  // (SEGS > 1: the workgroup's waves share a strip)
  const int grp = blockIdx.y, b = blockIdx.z;
  // one workgroup per sample clears the state of the selection that follows this kernel
  if (blockIdx.x == 0 && grp == 0) prep_sample(prep, b, threadIdx.x, WAVES * kWave);
  LanePos<D> p;
  int row0, col0;
  const bool active = locate<D, V4>(m, g, unit, p, row0, col0);
  const int c0 = grp * Cg, n_ch = min(C, c0 + Cg) - c0;
  // whole waves leave (SEGS > 1: the waves of a workgroup share their strip, and every segment
  // has lanes inside the plane, so they leave or stay together)
  if (__ballot(active) == 0 || n_ch <= 0) return;

  const int32_t *jm1 = jmap1 + (size_t)b * g.N;
  const bool up_in = row0 > 0, dn_in = row0 + (1 << D) < g.H;
  const ChainGeo<D> cg = chain_setup<D>(jm1, k1, p, active, up_in, dn_in, tiles[wv]);

  FwdSink<D, V4, false, SQ> sink;
#pragma unroll
  for (int s = 0; s < NS; ++s) sink.acc[s] = 0.f;
  if constexpr (FwdSink<D, V4, false, SQ>::MX) {
#pragma unroll
    for (int s = 0; s < NS; ++s) sink.top[s] = 0.f;
  }
  sink.plane = nullptr;
  chain_walk<D, SEGS>(yc1 + ((size_t)b * C + c0) * k1, k1, n_ch, wdw + (size_t)c0 * 9, cg, tiles[wv], p,
                      p.lc == 0, p.lc == m.lpr - 1 || col0 + V4 >= g.W, xchg, wv, sink,
                      [](FwdSink<D, V4, false, SQ> &) {});
  if (!active) return;
  write_slots<D, V4>(norm_part + ((size_t)grp * B + b) * g.N, sink.acc, p);
  if constexpr (FwdSink<D, V4, false, SQ>::MX) {
    if (max_part != nullptr) write_slots<D, V4>(max_part + ((size_t)grp * B + b) * g.N, sink.top, p);
  }
}

// ---- second pass: the kept coefficients of HWT(K_dw t1) ---------------------------------------------
// grid = (ceil(units/waves), G, B), block = waves = chain_waves(SEGS) waves.  jmap3: the consumer layer's rank map; xc
// [B, C, k3] fp32, or int8 codes with Q8 (clipping parameter: q_alpha > 0, or the largest of the
// n_alpha floats at alpha_src; the first workgroup leaves it at alpha_pub[0]).  Without Q8 the
// alpha slots (nullable) are raised to max |kept coefficient|.
template <int D, bool Q8, int SEGS>
__global__ __launch_bounds__(chain_waves(SEGS) * kWave, 4 / chain_waves(SEGS)) void chain_keep_kernel(const float *__restrict__ yc1,
                                                         const int32_t *__restrict__ jmap1,
                                                         int64_t k1, const float *__restrict__ wdw,
                                                         const int32_t *__restrict__ jmap3,
                                                         void *__restrict__ xc, int64_t k3,
                                                         float *alpha_slots, Geo g, StripMap m,
                                                         int C, int Cg, float q_alpha,
                                                         const float *__restrict__ alpha_src,
                                                         int n_alpha, float *alpha_pub) {
  constexpr int NS = slot_count(D, V4), WAVES = chain_waves(SEGS);
  __shared__ __attribute__((aligned(16))) uint32_t tiles[WAVES][ChainTiles<D>::kWords];
  __shared__ float xchg[ChainXchg<D, SEGS>::kWords];
  __shared__ float wmax[WAVES];
  const int wv = threadIdx.x >> 6;
  const int unit = blockIdx.x * WAVES + wv;
  const int grp = blockIdx.y, b = blockIdx.z;
  LanePos<D> p;
  int row0, col0;
  const bool active = locate<D, V4>(m, g, unit, p, row0, col0);
  const int c0 = grp * Cg, n_ch = max(min(C, c0 + Cg) - c0, 0);

  using Sink = KeepSink<D, V4, Q8>;
  using Out = typename Sink::Out;
  Sink sink(0.f);
  // the consumer's ranks of this lane's positions (or -1)
  const int32_t *jm3 = jmap3 + (size_t)b * g.N;
  auto fetch = [&](auto Lc, auto Jc) {
    constexpr int L = decltype(Lc)::value, J = decltype(Jc)::value;
    constexpr int CV = cols_at(V4, L), S2 = span_at(V4, L);
    const bool owner = (S2 == 1) || ((p.lc & (S2 - 1)) == 0);
#pragma unroll
    for (int i = 0; i < rows_at(D, L); ++i)
#pragma unroll
      for (int e = 0; e < CV; ++e) {
        int j = -1;
        if (active && owner) j = jm3[J * p.nl[L] + p.off[L] + i * p.rowlen[L] + e];
        sink.at[slot_base(D, V4, L, J) + i * CV + e] = (uint32_t)j;
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

  // The consumer's packed list of kept positions of this strip (rank, cell of the lane's own
  // slot), slot-major, then lane: built in the tile before the producer's list takes it over.
  constexpr int kRankBits = kInvRankBits;
  constexpr int STRIDE = ChainGeo<D>::STRIDE;
  uint32_t *tile = tiles[wv];
  const int lane = threadIdx.x & (kWave - 1);
  int count3 = 0;
#pragma unroll
  for (int s = 0; s < NS; ++s) count3 += __popcll(__ballot((int)sink.at[s] >= 0));
  const bool listed3 = count3 <= 16 * kWave && k3 <= ((int64_t)1 << kRankBits);
  uint32_t cell3[16], at3[16];  // this lane's share: entries lane + 64 i (unused rows fold away)
  if (listed3) {
    int running = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int j = (int)sink.at[s];
      const uint64_t kept = __ballot(j >= 0);
      const int to = running + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(kept >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)kept, 0u));
      if (j >= 0) tile[to] = (uint32_t)j | ((uint32_t)(lane * STRIDE + s) << kRankBits);
      running += __popcll(kept);
    }
    wave_lds_fence();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int e = lane + kWave * i;
      const uint32_t packed = e < count3 ? tile[e] : 0u;
      cell3[i] = e < count3 ? packed >> kRankBits : (uint32_t)(lane * STRIDE);
      at3[i] = e < count3 ? (packed & ((1u << kRankBits) - 1u)) * (uint32_t)sizeof(Out) : Sink::kDropped;
    }
    wave_lds_fence();
  }

  const int32_t *jm1 = jmap1 + (size_t)b * g.N;
  const bool up_in = row0 > 0, dn_in = row0 + (1 << D) < g.H;
  const ChainGeo<D> cg = chain_setup<D>(jm1, k1, p, active, up_in, dn_in, tile);

  if constexpr (Q8) {
    if (alpha_src != nullptr) {  // (uniform over the grid; every thread of the workgroup is here)
      q_alpha = alpha_max(alpha_src, n_alpha);
      if (alpha_pub != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
        alpha_pub[0] = q_alpha;
    }
  }

  float mx = 0.f;  // the wave's largest |kept coefficient| (fp32 output only)
  if (__ballot(active) != 0 && n_ch > 0) {
    Out *plane3 = static_cast<Out *>(xc) + ((size_t)b * C + c0) * k3;
    const float *plane1 = yc1 + ((size_t)b * C + c0) * k1;
    const float *kw = wdw + (size_t)c0 * 9;
    const bool first_lane = p.lc == 0, last_lane = p.lc == m.lpr - 1 || col0 + V4 >= g.W;
    // Both lists short enough: dense stores of the consumer's list (NI3 rows), producer's list
    // walked with NI1 rows.  The two go together (both layers keep the same fraction), so three
    // pairs cover the cases instead of every combination.
    auto staged = [&](auto ni3_c, auto ni1_c) {
      constexpr int NI3 = decltype(ni3_c)::value, NI1 = decltype(ni1_c)::value;
      ChainStagedSink<D, Q8, NI3> st(Q8 ? q_alpha : 0.f);
      st.tile = tile;
      st.row = tile + lane * STRIDE;
#pragma unroll
      for (int i = 0; i < NI3; ++i) { st.cell[i] = cell3[i]; st.at[i] = at3[i]; }
      st.vmax = 0.f;
      st.aim(plane3, k3);
      chain_walk<D, SEGS, NI1>(plane1, k1, n_ch, kw, cg, tile, p, first_lane,
                         last_lane, xchg, wv, st, [&plane3, k3](auto &sk) {
                           sk.flush();
                           plane3 += k3;
                           sk.aim(plane3, k3);
                         });
      mx = st.vmax;
    };
    const int ni3 = (count3 + kWave - 1) >> 6, ni1 = (cg.count + kWave - 1) >> 6;
    if (listed3 && cg.packed && cg.count > 0 && ni3 <= 4 && ni1 <= 8) {
      staged(std::integral_constant<int, 4>{}, std::integral_constant<int, 8>{});
    } else if (listed3 && cg.packed && cg.count > 0 && ni3 <= 8 && ni1 <= 16) {
      staged(std::integral_constant<int, 8>{}, std::integral_constant<int, 16>{});
    } else if (listed3 && cg.packed && cg.count > 0 && ni3 <= 16 && ni1 <= 32) {
      staged(std::integral_constant<int, 16>{}, std::integral_constant<int, 32>{});
    } else {
      // one store per slot (lanes that keep nothing there aim beyond the vector)
      if constexpr (Q8) sink.quant = Quant(q_alpha);
#pragma unroll
      for (int s = 0; s < NS; ++s)
        sink.at[s] = (int)sink.at[s] >= 0 ? sink.at[s] * (uint32_t)sizeof(Out) : Sink::kDropped;
      sink.vmax = 0.f;
      sink.aim(plane3, k3);
      // (a second sink with the quantiser's division path fixed at compile time, as in
      // haar_keep.hip, was measured here and lost: 761 vs 571 us on 96-wide planes -- this kernel
      // is short of registers as it is)
      chain_walk<D, SEGS>(plane1, k1, n_ch, kw, cg, tile, p, first_lane, last_lane, xchg, wv,
                    sink, [&plane3, k3](Sink &sk) {
                      plane3 += k3;
                      sk.aim(plane3, k3);
                    });
      mx = sink.vmax;
    }
  }
  if constexpr (Q8) return;
  if (alpha_slots == nullptr) return;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  if ((threadIdx.x & 63) == 0) wmax[wv] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    mx = wmax[0];
#pragma unroll
    for (int i = 1; i < WAVES; ++i) mx = fmaxf(mx, wmax[i]);
    unsigned int *a = reinterpret_cast<unsigned int *>(alpha_slots) +
                      ((blockIdx.x + 3u * blockIdx.y + 11u * blockIdx.z) & (kAlphaSlots - 1));
    const unsigned int mine = __float_as_uint(mx);
    if (mine > __hip_atomic_load(a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(a, mine);
  }
}

}  // namespace

// How the chained passes tile a plane: as the other strip kernels do where a wave row holds a
// whole row of the plane; else full wave rows side by side (one strip a wave, ceil(W/256) segments).
static StripMap chain_map(const wcc_desc &d) {
  StripMap m = make_map(d, V4);
  if (dw_needs_edges(m)) {
    m.lpr = kWave;
    m.log_lpr = 6;
    m.col_segs = (m.lanes_w + kWave - 1) / kWave;
    m.units = m.strips * m.col_segs;
  }
  return m;
}

// Segments of a row (waves that share it): 1 if a wave row holds the whole row, else 2 or 4;
// 0: a shape the chained passes do not take.
static int chain_segments(const wcc_desc &d) {
  if (d.W % 4 != 0 || d.levels > 3) return 0;
  const StripMap m = chain_map(d);
  if (!dw_needs_edges(m)) return 1;
  return (m.col_segs == 2 || m.col_segs == 4) ? m.col_segs : 0;
}

// Can the project layer d take its input from a producer's compressed output (see the limits at
// the top of this file)?
bool chain_supported(const wcc_desc &d) { return chain_segments(d) != 0; }

hipError_t launch_chain_norm(const wcc_desc &d, const ChainSrc &src, const float *wdw,
                             float *norm_part, float *max_part, int G, const SelectPrep &prep,
                             hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = chain_map(d);
  const int Cg = (d.C_in + G - 1) / G;
  const int segs = chain_segments(d), waves = chain_waves(segs);
  if (segs == 0) return hipErrorInvalidValue;
  const dim3 grid((m.units + waves - 1) / waves, G, d.B), block(waves * kWave);
  const bool sq = d.norm == WCC_NORM_L2;
#define WCC_CHAIN_NORM_(D_, SQ_, S_)                                                                   \
  hipLaunchKernelGGL((chain_norm_kernel<D_, SQ_, S_>), grid, block, 0, s, src.yc, src.jmap, src.k, wdw, \
                     norm_part, max_part, g, m, d.C_in, Cg, d.B, prep)
#define WCC_CHAIN_NORM(D_)                                                \
  do {                                                                    \
    if (segs == 1) {                                                      \
      if (sq) WCC_CHAIN_NORM_(D_, true, 1); else WCC_CHAIN_NORM_(D_, false, 1); \
    } else if (segs == 2) {                                               \
      if (sq) WCC_CHAIN_NORM_(D_, true, 2); else WCC_CHAIN_NORM_(D_, false, 2); \
    } else {                                                              \
      if (sq) WCC_CHAIN_NORM_(D_, true, 4); else WCC_CHAIN_NORM_(D_, false, 4); \
    }                                                                     \
  } while (0)
  switch (d.levels) {
    case 1: WCC_CHAIN_NORM(1); break;
    case 2: WCC_CHAIN_NORM(2); break;
    case 3: WCC_CHAIN_NORM(3); break;
    default: return hipErrorInvalidValue;
  }
#undef WCC_CHAIN_NORM
#undef WCC_CHAIN_NORM_
  return hipGetLastError();
}

hipError_t launch_chain_keep(const wcc_desc &d, int64_t k, const ChainSrc &src, const float *wdw,
                             const int32_t *jmap, void *xc, float *alpha_slots, float q_alpha,
                             const float *alpha_src, int n_alpha, float *alpha_pub, hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = chain_map(d);
  const int G = groups_for(d, d.C_in, 4096, 8);
  const int Cg = (d.C_in + G - 1) / G;
  const int segs = chain_segments(d), waves = chain_waves(segs);
  if (segs == 0) return hipErrorInvalidValue;
  const dim3 grid((m.units + waves - 1) / waves, G, d.B), block(waves * kWave);
  const bool q8 = q_alpha > 0.f || alpha_src != nullptr;
#define WCC_CHAIN_KEEP_(D_, S_)                                                                     \
  do {                                                                                              \
    if (q8)                                                                                         \
      hipLaunchKernelGGL((chain_keep_kernel<D_, true, S_>), grid, block, 0, s, src.yc, src.jmap,    \
                         src.k, wdw, jmap, xc, k, nullptr, g, m, d.C_in, Cg, q_alpha, alpha_src,    \
                         n_alpha, alpha_pub);                                                       \
    else                                                                                            \
      hipLaunchKernelGGL((chain_keep_kernel<D_, false, S_>), grid, block, 0, s, src.yc, src.jmap,   \
                         src.k, wdw, jmap, xc, k, alpha_slots, g, m, d.C_in, Cg, 0.f, nullptr, 0,   \
                         nullptr);                                                                  \
  } while (0)
#define WCC_CHAIN_KEEP(D_)                     \
  do {                                         \
    if (segs == 1) WCC_CHAIN_KEEP_(D_, 1);     \
    else if (segs == 2) WCC_CHAIN_KEEP_(D_, 2); \
    else WCC_CHAIN_KEEP_(D_, 4);               \
  } while (0)
  switch (d.levels) {
    case 1: WCC_CHAIN_KEEP(1); break;
    case 2: WCC_CHAIN_KEEP(2); break;
    case 3: WCC_CHAIN_KEEP(3); break;
    default: return hipErrorInvalidValue;
  }
#undef WCC_CHAIN_KEEP
#undef WCC_CHAIN_KEEP_
  return hipGetLastError();
}

}  // namespace wcc
