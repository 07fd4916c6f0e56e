// Sources and sinks of the strip transform shared by its kernels: where the analysis puts its
// coefficients (channel norms, kept coefficients) and where the synthesis takes them from (the
// kept values of a compressed signal, everything else zero).
#pragma once
#include "strip.h"

namespace wcc {
namespace {

// ---- analysis ---------------------------------------------------------------------------
// STORE = false: only the |coefficient| sums are kept (the norm-only pass of the fused layer),
// and beside them the largest |coefficient| over the channels at every position: the largest
// of those over the positions the selection keeps is the layer's clipping parameter alpha, known
// that way before the second pass, which can then decide the 8-bit codes itself.
// SQ: the sums are of squared coefficients (one fused multiply-add each) instead.
template <int D, int V, bool STORE, bool SQ = false>
struct FwdSink {
  static constexpr bool MX = !STORE;
  float *plane;  // wavelet vector of the current (b, c)
  float acc[slot_count(D, V)];
  float top[MX ? slot_count(D, V) : 1];  // max over the channels of |coefficient|
  template <int L, int J>
  __device__ __forceinline__ void put_row(const LanePos<D> &p, int i, const float (&v)[cols_at(V, L)],
                                          bool owner) {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
#pragma unroll
    for (int e = 0; e < CV; ++e) {
      float &a = acc[base + i * CV + e];
      a = SQ ? fmaf(v[e], v[e], a) : a + fabsf(v[e]);
      if constexpr (MX) top[base + i * CV + e] = fmaxf(top[base + i * CV + e], fabsf(v[e]));
    }
    if (!STORE || !owner) return;
    float *dst = plane + (J * p.nl[L] + p.off[L] + i * p.rowlen[L]);
    if constexpr (CV == 2) {
      *reinterpret_cast<float2 *>(dst) = make_float2(v[0], v[1]);
    } else {
#pragma unroll
      for (int e = 0; e < CV; ++e) dst[e] = v[e];
    }
  }
};

// One value per slot of the lane's tile, written with the same addressing as the coefficients
// (np: a [N] plane in the order of the wavelet vector).  Lanes that do not own a slot's value
// skip it.
template <int D, int V>
__device__ __forceinline__ void write_slots(float *np, const float *vals, const LanePos<D> &p) {
  auto flush = [&](auto Lc, auto Jc) {
    constexpr int L = decltype(Lc)::value, J = decltype(Jc)::value;
    constexpr int CV = cols_at(V, L), S2 = span_at(V, L);
    const bool owner = (S2 == 1) || ((p.lc & (S2 - 1)) == 0);
    if (!owner) return;
#pragma unroll
    for (int i = 0; i < rows_at(D, L); ++i) {
      float *dst = np + (J * p.nl[L] + p.off[L] + i * p.rowlen[L]);
      if constexpr (CV == 2) {
        *reinterpret_cast<float2 *>(dst) = make_float2(vals[slot_base(D, V, L, J) + i * CV],
                                                       vals[slot_base(D, V, L, J) + i * CV + 1]);
      } else {
#pragma unroll
        for (int e = 0; e < CV; ++e) dst[e] = vals[slot_base(D, V, L, J) + i * CV + e];
      }
    }
  };
  auto each_level = [&](auto Lc) {
    constexpr int L = decltype(Lc)::value;
    flush(Lc, std::integral_constant<int, 1>{});
    flush(Lc, std::integral_constant<int, 2>{});
    flush(Lc, std::integral_constant<int, 3>{});
    if constexpr (L == D) flush(Lc, std::integral_constant<int, 0>{});
  };
  each_level(std::integral_constant<int, 1>{});
  if constexpr (D >= 2) each_level(std::integral_constant<int, 2>{});
  if constexpr (D >= 3) each_level(std::integral_constant<int, 3>{});
  if constexpr (D >= 4) each_level(std::integral_constant<int, 4>{});
}

// ---- second pass of the fused layer: transform again, keep only the selected positions ----
// xc[b, c, jmap[b, q]] = HWT_d(x[b, c])[q] for the kept q; dropped coefficients never reach
// memory.  Also raises the alpha slots to max |kept coefficient| (nullable).
// Q8: the clipping parameter is known beforehand (the caller supplied it), so the kept
// coefficients leave the chip as signed 8-bit codes (Eq. quantweights) instead of fp32.
// QF: which division the quantiser takes, 1 = the fast one, 2 = the IEEE divide (the caller has
// looked at Quant::fast once for the whole walk), 0 = looked up row by row.
template <int D, int V, bool Q8, int QF = 0>
struct KeepSink {
  using Out = std::conditional_t<Q8, int8_t, float>;
  // Every slot is stored through a buffer descriptor of the channel's compressed vector, with
  // the byte offset of the slot's rank, or an offset beyond the vector for a position that is
  // not kept: the hardware drops such a lane's store.  No store sits behind a branch, so the
  // number of stores per channel is fixed and the wait for the prefetched rows of the next
  // channel does not have to drain them (loads and stores retire through one counter); and no
  // slot needs a 64-bit address or a saved lane mask, which halves the kernel's registers.
  static constexpr uint32_t kDropped = 0xFFFFFFFFu;
  __amdgpu_buffer_rsrc_t xc_c;     // xc[b, c, :]
  uint32_t at[slot_count(D, V)];   // byte offset of the slot's rank, or kDropped
  float vmax;
  Quant quant;
  __device__ __forceinline__ explicit KeepSink(float alpha) : quant(alpha) {}
  template <int QF2>
  __device__ __forceinline__ explicit KeepSink(const KeepSink<D, V, Q8, QF2> &o)
      : xc_c(o.xc_c), vmax(o.vmax), quant(o.quant) {
#pragma unroll
    for (int s = 0; s < slot_count(D, V); ++s) at[s] = o.at[s];
  }
  // plane: xc[b, c, :] (wave-uniform), k elements
  __device__ __forceinline__ void aim(Out *plane, int64_t k) {
    xc_c = __builtin_amdgcn_make_buffer_rsrc(plane, 0, (int)(uint32_t)(k * (int64_t)sizeof(Out)),
                                             0x00020000 /* raw dwords, no swizzle */);
  }
  template <int L, int J>
  __device__ __forceinline__ void put_row(const LanePos<D> &p, int i, const float (&v)[cols_at(V, L)],
                                          bool owner) {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
    (void)p;
    (void)owner;  // (at[] is kDropped for the lanes that do not own the value)
    if constexpr (Q8) {
      // (the quantiser's division path is chosen once per row, not value by value)
      auto store_codes = [&](auto fast_c) {
        constexpr bool FAST = decltype(fast_c)::value;
#pragma unroll
        for (int e = 0; e < CV; ++e)
          __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(int8_t)(int)quant.template level_as<FAST>(v[e]),
                                               xc_c, at[base + i * CV + e], 0, 0);
      };
      if constexpr (QF == 1) store_codes(std::true_type{});
      else if constexpr (QF == 2) store_codes(std::false_type{});
      else if (quant.fast) store_codes(std::true_type{});
      else store_codes(std::false_type{});
    } else {
#pragma unroll
      for (int e = 0; e < CV; ++e) {
        const int s = base + i * CV + e;
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[e]), xc_c, at[s], 0, 0);
        vmax = fmaxf(vmax, at[s] != kDropped ? fabsf(v[e]) : 0.f);
      }
    }
  }
};

// The same sink for a strip that keeps few of its positions.  One sparse store per slot costs
// the memory pipeline an instruction each, whatever the number of lanes that keep something
// (measured: the stores were a third of the pass).  Here every lane drops its values into an LDS
// tile laid out [slot][lane]; after the last level the wave goes through the strip's packed list
// of kept positions (64 entries a row, built once, the same for every channel), picks each
// entry's value from the tile and stores NI dense rows instead of one row per slot.
template <int D, int V, bool Q8, int NI>
struct KeepStagedSink {
  using Out = std::conditional_t<Q8, int8_t, float>;
  static constexpr uint32_t kDropped = 0xFFFFFFFFu;
  __amdgpu_buffer_rsrc_t xc_c;  // xc[b, c, :]
  uint32_t *tile;               // [slot][lane]
  int lane;
  uint32_t cell[NI];            // tile index of the entry's position
  uint32_t at[NI];              // byte offset of the entry's rank, or kDropped (list padding)
  float vmax;
  Quant quant;
  __device__ __forceinline__ explicit KeepStagedSink(float alpha) : quant(alpha) {}
  __device__ __forceinline__ void aim(Out *plane, int64_t k) {
    xc_c = __builtin_amdgcn_make_buffer_rsrc(plane, 0, (int)(uint32_t)(k * (int64_t)sizeof(Out)),
                                             0x00020000 /* raw dwords, no swizzle */);
  }
  template <int L, int J>
  __device__ __forceinline__ void put_row(const LanePos<D> &p, int i, const float (&v)[cols_at(V, L)],
                                          bool owner) {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
    (void)p;
    (void)owner;  // (a value a lane does not own is in no list)
#pragma unroll
    for (int e = 0; e < CV; ++e) tile[(base + i * CV + e) * kWave + lane] = __float_as_uint(v[e]);
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
  }
};

// ---- synthesis sources ---------------------------------------------------------------------------
constexpr int kInvCap = 1024;          // packed entries per wave
constexpr uint32_t kInvNone = ~0u;     // list padding
constexpr int kInvRankBits = 20;       // entry = rank | cell << 20

// Plain path: jj[slot] = rank j of the position inside the kept list, or -1 (dropped -> 0);
// one conditional load per slot that some lane keeps.
template <int D, int V>
struct InvDirect {
  const float *plane;  // yc[b, o, :]
  int jj[slot_count(D, V)];
  uint64_t any[2];     // wave-uniform: bit s set if some lane keeps slot s
  template <int L, int J>
  __device__ __forceinline__ void get_row(int i, float (&v)[cols_at(V, L)]) const {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
#pragma unroll
    for (int e = 0; e < CV; ++e) {
      const int s = base + i * CV + e;
      float t = 0.f;
      if ((any[s >> 6] >> (s & 63)) & 1) {
        const int j = jj[s];
        if (j >= 0) t = plane[j];
      }
      v[e] = t;
    }
  }
};

// Staged: the lane's cell of the [slot][lane] LDS tile (zero unless the position is kept).
template <int D, int V>
struct InvStaged {
  const float *cell;   // &tile[0][lane]
  uint64_t any[2];     // wave-uniform: bit s set if some lane keeps slot s
  template <int L, int J>
  __device__ __forceinline__ void get_row(int i, float (&v)[cols_at(V, L)]) const {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
#pragma unroll
    for (int e = 0; e < CV; ++e) {
      const int s = base + i * CV + e;
      v[e] = ((any[s >> 6] >> (s & 63)) & 1) ? cell[s * kWave] : 0.f;
    }
  }
};

template <int D, int V, int L, class Source>
__device__ __forceinline__ void inv_levels(float (&out)[rows_at(D, L - 1)][cols_at(V, L - 1)],
                                           const LanePos<D> &p, const Source &src) {
  constexpr int R2 = rows_at(D, L), VI = cols_at(V, L - 1), V2 = cols_at(V, L);
  constexpr int SI = span_at(V, L - 1);
  float ll[R2][V2];
  if constexpr (L < D) {
    inv_levels<D, V, L + 1>(ll, p, src);
  } else {
#pragma unroll
    for (int i = 0; i < R2; ++i) src.template get_row<L, 0>(i, ll[i]);
  }
#pragma unroll
  for (int i = 0; i < R2; ++i) {
    float y2[V2], y3[V2], y4[V2];
    src.template get_row<L, 1>(i, y2);
    src.template get_row<L, 2>(i, y3);
    src.template get_row<L, 3>(i, y4);
#pragma unroll
    for (int e = 0; e < V2; ++e) {
      const float s1 = ll[i][e] + y3[e], s2 = ll[i][e] - y3[e];
      const float d1 = y2[e] + y4[e], d2 = y2[e] - y4[e];
      const float a = 0.5f * (s1 + d1), b = 0.5f * (s1 - d1);
      const float c = 0.5f * (s2 + d2), d = 0.5f * (s2 - d2);
      if constexpr (VI >= 2) {
        out[2 * i][2 * e] = a; out[2 * i][2 * e + 1] = b;
        out[2 * i + 1][2 * e] = c; out[2 * i + 1][2 * e + 1] = d;
      } else {
        // every lane of the group holds the same (y1..y4); the left half keeps the left pixel
        const bool left = (p.lc & SI) == 0;
        out[2 * i][0] = left ? a : b;
        out[2 * i + 1][0] = left ? c : d;
      }
    }
  }
}

// The wave's LDS tile is laid out [lane][slot]: a lane's NT slots are contiguous, so one channel's
// kept values come back with NT / 4 16-byte reads and no branch (cells of positions that are
// not kept hold zero).  The lane stride is an odd multiple of four words: the 16 lanes of one
// read cycle then touch every bank once.
__host__ __device__ constexpr int tile_stride(int nt) { return (nt / 4) % 2 == 1 ? nt : nt + 4; }

// sources of the synthesis: the lane's slots as read back from the tile into registers
template <int D, int V, int N>
struct RegStrip {
  const float (&c)[N];
  template <int L, int J>
  __device__ __forceinline__ void get_row(int i, float (&v)[cols_at(V, L)]) const {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
#pragma unroll
    for (int e = 0; e < CV; ++e) v[e] = c[base + i * CV + e];
  }
};
}  // namespace
}  // namespace wcc
