// Shared by the three transform translation units (haar_fwd.hip, haar_keep.hip,
// haar_inv.hip): the register-resident strip transform and how waves tile a plane.
//
// Multi-level Haar analysis / synthesis for gfx950 (Eq. HaarKernel, Eq. wavelet_transform; the
// inverse undoes the levels last to first with the transposed kernels), with the channel L1 norm
// of Alg. 1 fused into the analysis and the zero filling T^T fused into the synthesis.
//
// Design.  A d-level Haar transform is local to 2^d x 2^d pixel blocks, so the whole
// transform of a strip of 2^d image rows can live in registers: all levels cost one HBM read
// and one HBM write.  A lane owns V = 4 adjacent columns of the strip (one 16-byte load per
// row); a wavefront therefore reads 1 KiB-contiguous row segments.  Levels 1 and 2 pair
// columns inside the lane; from level 3 on the horizontal partner is the lane at distance
// 1, 2, ... and is reached with a DPP quad permute -- no LDS is needed.  The values a wave
// produces for one band row are contiguous in the wavelet vector, so every store is a
// contiguous run as well (8 bytes per lane at level 1, 4 at level 2, ...).
// Each wave walks a group of channels over the same strip, prefetching the next channel's
// rows while it transforms the current one; per-position |coefficient| sums stay in
// registers and are written once per channel group.
#pragma once
#include <type_traits>

#include "wcc_internal.h"

namespace wcc {
namespace {

// ---- compile-time shape of the per-lane tile at every level --------------------------------
// level 0 tile: (1<<D) rows x V columns.  Going to level l halves the rows; it halves the
// columns while there are >= 2 in the lane, afterwards it doubles the "span" (number of
// lanes that hold the same value).
__host__ __device__ constexpr int cols_at(int V, int l) { return (V >> l) > 0 ? (V >> l) : 1; }
__host__ __device__ constexpr int span_at(int V, int l) {
  int s = 1, v = V;
  for (int i = 0; i < l; ++i) {
    if (v >= 2) v /= 2; else s *= 2;
  }
  return s;
}
__host__ __device__ constexpr int rows_at(int D, int l) { return 1 << (D - l); }
// register slot of (level l, band j, row i, column e); band 0 exists only at level D
__host__ __device__ constexpr int slot_base(int D, int V, int l, int j) {
  int s = 0;
  for (int m = 1; m < l; ++m) s += 3 * rows_at(D, m) * cols_at(V, m);
  if (l == D) return s + j * rows_at(D, l) * cols_at(V, l);  // 4 bands at the last level
  return s + (j - 1) * rows_at(D, l) * cols_at(V, l);
}
__host__ __device__ constexpr int slot_count(int D, int V) {
  return slot_base(D, V, D, 3) + rows_at(D, D) * cols_at(V, D);
}

template <int S>
__device__ __forceinline__ float lane_xor(float v) {
  int x = __float_as_int(v);
  if constexpr (S == 1) {
    x = __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
  } else if constexpr (S == 2) {
    x = __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
  } else {
    x = __shfl_xor(x, S, kWave);
  }
  return __int_as_float(x);
}

// Where a lane's values of every level land inside one plane's wavelet vector.
template <int D>
struct LanePos {
  int off[D + 1];     // off[l]: (first row >> l) * (W >> l) + (first column >> l), l = 1..D
  int rowlen[D + 1];  // W >> l
  int nl[D + 1];      // band size n_l
  int lc;             // lane's column index inside its row of lanes
  bool active;        // lane maps to pixels of the plane
};

template <int D, int V, int L, class Sink>
__device__ __forceinline__ void fwd_levels(const float (&in)[rows_at(D, L - 1)][cols_at(V, L - 1)],
                                           const LanePos<D> &p, Sink &sink) {
  constexpr int R2 = rows_at(D, L), VI = cols_at(V, L - 1), V2 = cols_at(V, L);
  constexpr int SI = span_at(V, L - 1), S2 = span_at(V, L);
  float ll[R2][V2];
  const bool owner = p.active && ((S2 == 1) || ((p.lc & (S2 - 1)) == 0));
#pragma unroll
  for (int i = 0; i < R2; ++i) {
    float y2[V2], y3[V2], y4[V2];
#pragma unroll
    for (int e = 0; e < V2; ++e) {
      float a, b, c, d;
      if constexpr (VI >= 2) {
        a = in[2 * i][2 * e]; b = in[2 * i][2 * e + 1];
        c = in[2 * i + 1][2 * e]; d = in[2 * i + 1][2 * e + 1];
      } else {
        const float o0 = in[2 * i][0], o1 = in[2 * i + 1][0];
        const float q0 = lane_xor<SI>(o0), q1 = lane_xor<SI>(o1);
        const bool left = (p.lc & SI) == 0;
        a = left ? o0 : q0; b = left ? q0 : o0;
        c = left ? o1 : q1; d = left ? q1 : o1;
      }
      const float s1 = a + b, s2 = c + d, d1 = a - b, d2 = c - d;
      ll[i][e] = 0.5f * (s1 + s2);
      y2[e] = 0.5f * (d1 + d2);
      y3[e] = 0.5f * (s1 - s2);
      y4[e] = 0.5f * (d1 - d2);
    }
    sink.template put_row<L, 1>(p, i, y2, owner);
    sink.template put_row<L, 2>(p, i, y3, owner);
    sink.template put_row<L, 3>(p, i, y4, owner);
    if constexpr (L == D) sink.template put_row<L, 0>(p, i, ll[i], owner);
  }
  if constexpr (L < D) fwd_levels<D, V, L + 1>(ll, p, sink);
}

template <int V> struct VecT;
template <> struct VecT<4> { using type = float4; };
template <> struct VecT<2> { using type = float2; };

template <int V>
__device__ __forceinline__ void load_row(const float *src, float (&dst)[V]) {
  using T = typename VecT<V>::type;
  const T t = *reinterpret_cast<const T *>(src);
  dst[0] = t.x; dst[1] = t.y;
  if constexpr (V == 4) { dst[2] = t.z; dst[3] = t.w; }
}
template <int V>
__device__ __forceinline__ void store_row(float *dst, const float (&src)[V]) {
  using T = typename VecT<V>::type;
  T t;
  t.x = src[0]; t.y = src[1];
  if constexpr (V == 4) { t.z = src[2]; t.w = src[3]; }
  *reinterpret_cast<T *>(dst) = t;
}
__device__ __forceinline__ float load_one(const float *src) { return *src; }

// Streaming variants: the access carries the non-temporal hint, so it does not claim lines in
// the memory-side cache.  Used for tensors much larger than that cache that are read or written
// once: without the hint the output of the inverse transform fills the cache with dirty lines
// whose write-back the next reader of anything pays for.
typedef float stream_f4 __attribute__((ext_vector_type(4)));
typedef float stream_f2 __attribute__((ext_vector_type(2)));
typedef uint32_t stream_u2 __attribute__((ext_vector_type(2)));
template <int V>
__device__ __forceinline__ void load_row_stream(const float *src, float (&dst)[V]) {
  if constexpr (V == 4) {
    const stream_f4 t = __builtin_nontemporal_load(reinterpret_cast<const stream_f4 *>(src));
    dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
  } else {
    const stream_f2 t = __builtin_nontemporal_load(reinterpret_cast<const stream_f2 *>(src));
    dst[0] = t.x; dst[1] = t.y;
  }
}
template <int V>
__device__ __forceinline__ void store_row_stream(float *dst, const float (&src)[V]) {
  if constexpr (V == 4) {
    stream_f4 t;
    t.x = src[0]; t.y = src[1]; t.z = src[2]; t.w = src[3];
    __builtin_nontemporal_store(t, reinterpret_cast<stream_f4 *>(dst));
  } else {
    stream_f2 t;
    t.x = src[0]; t.y = src[1];
    __builtin_nontemporal_store(t, reinterpret_cast<stream_f2 *>(dst));
  }
}

// The same for activations stored as bf16 (bit patterns in uint16): widening is exact, narrowing
// rounds to nearest even.
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }
// two floats -> two bf16 in one word (first one in the low half), round to nearest even: one
// v_cvt_pk_bf16_f32 on this chip
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
template <int V>
__device__ __forceinline__ void load_row(const bf16_t *src, float (&dst)[V]) {
  if constexpr (V == 4) {
    const uint2 t = *reinterpret_cast<const uint2 *>(src);
    dst[0] = bf16_lo(t.x); dst[1] = bf16_hi(t.x); dst[2] = bf16_lo(t.y); dst[3] = bf16_hi(t.y);
  } else {
    const uint32_t t = *reinterpret_cast<const uint32_t *>(src);
    dst[0] = bf16_lo(t); dst[1] = bf16_hi(t);
  }
}
template <int V>
__device__ __forceinline__ void store_row(bf16_t *dst, const float (&src)[V]) {
  const uint32_t a = pack_bf16(src[0], src[1]);
  if constexpr (V == 4) {
    const uint32_t b = pack_bf16(src[2], src[3]);
    *reinterpret_cast<uint2 *>(dst) = make_uint2(a, b);
  } else {
    *reinterpret_cast<uint32_t *>(dst) = a;
  }
}
__device__ __forceinline__ float load_one(const bf16_t *src) { return __uint_as_float((uint32_t)*src << 16); }
template <int V>
__device__ __forceinline__ void load_row_stream(const bf16_t *src, float (&dst)[V]) {
  if constexpr (V == 4) {
    const stream_u2 t = __builtin_nontemporal_load(reinterpret_cast<const stream_u2 *>(src));
    dst[0] = bf16_lo(t.x); dst[1] = bf16_hi(t.x); dst[2] = bf16_lo(t.y); dst[3] = bf16_hi(t.y);
  } else {
    const uint32_t t = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(src));
    dst[0] = bf16_lo(t); dst[1] = bf16_hi(t);
  }
}
template <int V>
__device__ __forceinline__ void store_row_stream(bf16_t *dst, const float (&src)[V]) {
  const uint32_t a = pack_bf16(src[0], src[1]);
  if constexpr (V == 4) {
    stream_u2 t;
    t.x = a;
    t.y = pack_bf16(src[2], src[3]);
    __builtin_nontemporal_store(t, reinterpret_cast<stream_u2 *>(dst));
  } else {
    __builtin_nontemporal_store(a, reinterpret_cast<uint32_t *>(dst));
  }
}

// Rows through a buffer descriptor of one plane (non-temporal): the lane gives a byte offset
// into the plane, and an offset at or beyond the descriptor's size makes the hardware drop the
// store (return zeros for the load) without touching memory.  Lanes that stand outside the
// plane use that instead of a lane mask or a dummy target (a line of memory shared by all idle
// lanes of the chip turns into a hot spot: with 24 of 32 lanes a row in use it tripled the
// inverse's time).
constexpr uint32_t kRowDropped = 0xFFFFFFF0u;  // beyond any plane (H * W <= 2^30 - 16 elements)
constexpr int kBufStream = 2;                  // cache policy of the access: non-temporal
typedef uint32_t buf_u4 __attribute__((ext_vector_type(4)));
typedef uint32_t buf_u2 __attribute__((ext_vector_type(2)));
template <class YT>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t plane_rsrc(const YT *plane, int64_t n) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<YT *>(plane), 0, (int)(uint32_t)(n * (int64_t)sizeof(YT)),
                                           0x00020000 /* raw dwords, no swizzle */);
}
template <int V>
__device__ __forceinline__ void store_row_buf(__amdgpu_buffer_rsrc_t rsrc, uint32_t off,
                                              const float (&src)[V], float) {
  if constexpr (V == 4) {
    buf_u4 t = {__float_as_uint(src[0]), __float_as_uint(src[1]), __float_as_uint(src[2]), __float_as_uint(src[3])};
    __builtin_amdgcn_raw_buffer_store_b128(t, rsrc, off, 0, kBufStream);
  } else {
    buf_u2 t = {__float_as_uint(src[0]), __float_as_uint(src[1])};
    __builtin_amdgcn_raw_buffer_store_b64(t, rsrc, off, 0, kBufStream);
  }
}
template <int V>
__device__ __forceinline__ void store_row_buf(__amdgpu_buffer_rsrc_t rsrc, uint32_t off,
                                              const float (&src)[V], bf16_t) {
  const uint32_t a = pack_bf16(src[0], src[1]);
  if constexpr (V == 4) {
    buf_u2 t = {a, pack_bf16(src[2], src[3])};
    __builtin_amdgcn_raw_buffer_store_b64(t, rsrc, off, 0, kBufStream);
  } else {
    __builtin_amdgcn_raw_buffer_store_b32(a, rsrc, off, 0, kBufStream);
  }
}
template <int V>
__device__ __forceinline__ void load_row_buf(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, float (&dst)[V],
                                             float) {
  if constexpr (V == 4) {
    const buf_u4 t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, kBufStream);
    dst[0] = __uint_as_float(t.x); dst[1] = __uint_as_float(t.y);
    dst[2] = __uint_as_float(t.z); dst[3] = __uint_as_float(t.w);
  } else {
    const buf_u2 t = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, kBufStream);
    dst[0] = __uint_as_float(t.x); dst[1] = __uint_as_float(t.y);
  }
}
template <int V>
__device__ __forceinline__ void load_row_buf(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, float (&dst)[V],
                                             bf16_t) {
  if constexpr (V == 4) {
    const buf_u2 t = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, kBufStream);
    dst[0] = bf16_lo(t.x); dst[1] = bf16_hi(t.x); dst[2] = bf16_lo(t.y); dst[3] = bf16_hi(t.y);
  } else {
    const uint32_t t = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, kBufStream);
    dst[0] = bf16_lo(t); dst[1] = bf16_hi(t);
  }
}

// What a lane loads of one row, kept as it arrives: the widening of bf16 happens when the
// values are used, not where the load is issued (a conversion next to the load would wait for it
// and undo the prefetch).
template <int V, class T> struct Row;
template <int V> struct Row<V, float> {
  float v[V];
  template <bool NT = false>
  __device__ __forceinline__ void load(const float *src) {
    if constexpr (NT) load_row_stream<V>(src, v); else load_row<V>(src, v);
  }
  __device__ __forceinline__ void get(float (&d)[V]) const {
#pragma unroll
    for (int e = 0; e < V; ++e) d[e] = v[e];
  }
};
template <int V> struct Row<V, bf16_t> {
  uint32_t w[V / 2];
  template <bool NT = false>
  __device__ __forceinline__ void load(const bf16_t *src) {
    if constexpr (V == 4) {
      if constexpr (NT) {
        const stream_u2 t = __builtin_nontemporal_load(reinterpret_cast<const stream_u2 *>(src));
        w[0] = t.x; w[1] = t.y;
      } else {
        const uint2 t = *reinterpret_cast<const uint2 *>(src);
        w[0] = t.x; w[1] = t.y;
      }
    } else {
      w[0] = NT ? __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(src))
                : *reinterpret_cast<const uint32_t *>(src);
    }
  }
  __device__ __forceinline__ void get(float (&d)[V]) const {
#pragma unroll
    for (int e = 0; e < V / 2; ++e) { d[2 * e] = bf16_lo(w[e]); d[2 * e + 1] = bf16_hi(w[e]); }
  }
};

// How waves tile one plane.
struct StripMap {
  int lpr;        // lanes per strip row (power of two <= 64)
  int log_lpr;
  int col_segs;   // 64-lane column segments per row (1 unless lpr == 64)
  int lanes_w;    // W / V lanes needed per row
  int strips;     // H >> D
  int units;      // wave work items per plane
};

template <int D, int V>
__device__ __forceinline__ bool locate(const StripMap &m, const Geo &g, int unit, LanePos<D> &p,
                                       int &row0, int &col0) {
  const int lane = threadIdx.x & (kWave - 1);
  const int sub = lane >> m.log_lpr;
  p.lc = lane & (m.lpr - 1);
  const int ru = unit / m.col_segs, cs = unit - ru * m.col_segs;
  const int strip = ru * (kWave >> m.log_lpr) + sub;
  const int col_lane = cs * m.lpr + p.lc;
  row0 = strip << D;
  col0 = col_lane * V;
#pragma unroll
  for (int l = 1; l <= D; ++l) {
    p.rowlen[l] = g.W >> l;
    p.nl[l] = (g.H >> l) * (g.W >> l);
    p.off[l] = (row0 >> l) * p.rowlen[l] + (col0 >> l);
  }
  p.active = unit < m.units && strip < m.strips && col_lane < m.lanes_w;
  return p.active;
}

// Walks n_ch channel planes (stride N floats) of one strip: loads run PF channels ahead of the
// arithmetic, in a ring of PF + 1 register tiles.  after(sink) runs once per channel.
// Inside the main loop every step issues its prefetch and there is no branch: the number of
// outstanding loads must be the same on every path, or the wait in front of the arithmetic
// has to drain the prefetch as well (the counter is in order).  A prefetch past the last
// channel reads the last channel again (a cache hit); the at most PF channels left after the
// main loop are already in registers.
template <int D, int V, int PF, bool NT, class XT, class Sink, class After>
__device__ __forceinline__ void channel_loop(const XT *__restrict__ src, int64_t N, int W,
                                             int n_ch, const LanePos<D> &p, Sink &sink,
                                             After &&after) {
  constexpr int R = 1 << D;
  Row<V, XT> buf[PF + 1][R];
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const XT *nx = src + (size_t)min(u, n_ch - 1) * N;
#pragma unroll
    for (int r = 0; r < R; ++r) buf[u][r].template load<NT>(nx + (size_t)r * W);
  }
  int c = 0;
  for (; c + PF < n_ch; c += PF + 1) {
#pragma unroll
    for (int u = 0; u <= PF; ++u) {
      const XT *nx = src + (size_t)min(c + u + PF, n_ch - 1) * N;
#pragma unroll
      for (int r = 0; r < R; ++r) buf[(u + PF) % (PF + 1)][r].template load<NT>(nx + (size_t)r * W);
      __builtin_amdgcn_sched_barrier(0);  // the loads go out before the arithmetic, not after
      float in[R][V];
#pragma unroll
      for (int r = 0; r < R; ++r) buf[u][r].get(in[r]);
      fwd_levels<D, V, 1>(in, p, sink);
      after(sink);
    }
  }
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    if (c + u < n_ch) {
      float in[R][V];
#pragma unroll
      for (int r = 0; r < R; ++r) buf[u][r].get(in[r]);
      fwd_levels<D, V, 1>(in, p, sink);
      after(sink);
    }
  }
}

// ---- the same walk with a depthwise 3x3 convolution in front of the transform --------------
// (the paper's third ingredient: consecutive separable operations fused, so the convolved
// tensor is never written).  The transform's input tile is K_dw applied to the 2^d + 2 rows
// x (V + 2) columns around it: cross-correlation, zero padding 1, the same order of
// multiply-adds as the stand-alone kernel in depthwise.hip, so both give the same bits.
// The two columns outside a lane's V come from the neighbouring lanes' rows through a lane
// shuffle; the first and last lane of a wave row take theirs from memory (EDGE) or, where that
// is the border of the plane, zero.  Every load is issued on every path: rows above / below the
// plane and edge columns that do not exist are read from a valid address and masked.
struct DwLane {
  int row_step;       // W
  int top_step;       // offset of the row above the strip relative to its first row: -W or 0
  int bot_step;       // offset of the row below relative to the first row: R*W or (R-1)*W
  bool top_in, bot_in;
  bool first, last;   // lane is the first / last of its wave row (or the last one inside the plane)
  int left_off, right_off;  // EDGE: element offsets of the outside columns (0: none to read)
};

template <int D, int V>
__device__ __forceinline__ DwLane dw_lane(const Geo &g, const StripMap &m, const LanePos<D> &p,
                                          int row0, int col0) {
  constexpr int R = 1 << D;
  DwLane q;
  q.row_step = g.W;
  q.top_in = row0 > 0;
  q.bot_in = row0 + R < g.H;
  q.top_step = q.top_in ? -g.W : 0;
  q.bot_step = q.bot_in ? R * g.W : (R - 1) * g.W;
  q.first = p.lc == 0;
  q.last = p.lc == m.lpr - 1 || col0 + V >= g.W;
  q.left_off = (q.first && col0 > 0) ? -1 : 0;
  q.right_off = (q.last && col0 + V < g.W) ? V : 0;
  return q;
}

template <int D, int V, bool EDGE, bool PEEL, bool NT, class XT, class Sink, class After>
__device__ __forceinline__ void channel_loop_dw(const XT *__restrict__ src,
                                                const float *__restrict__ wdw, int64_t N, int n_ch,
                                                const DwLane &q, const LanePos<D> &p, Sink &sink,
                                                After &&after) {
  constexpr int R = 1 << D, RR = R + 2;
  Row<V, XT> raw[2][RR];
  XT el[2][EDGE ? RR : 1], er[2][EDGE ? RR : 1];  // outside columns, as stored
  auto row_ptr = [&](const XT *plane, int i) -> const XT * {
    return i == 0 ? plane + q.top_step : i == RR - 1 ? plane + q.bot_step
                                                     : plane + (size_t)(i - 1) * q.row_step;
  };
  auto load_tile = [&](int u, int ch) {
    const XT *plane = src + (size_t)min(ch, n_ch - 1) * N;
#pragma unroll
    for (int i = 0; i < RR; ++i) {
      const XT *rp = row_ptr(plane, i);
      raw[u][i].template load<NT>(rp);
      if constexpr (EDGE) {
        el[u][i] = rp[q.left_off];
        er[u][i] = rp[q.right_off];
      }
    }
  };
  auto transform = [&](int u, int ch) {
    float k[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) k[t] = wdw[(size_t)ch * 9 + t];
    float six[RR][V + 2];
#pragma unroll
    for (int i = 0; i < RR; ++i) {
      const bool in = i == 0 ? q.top_in : i == RR - 1 ? q.bot_in : true;
      float own[V];
      raw[u][i].get(own);
#pragma unroll
      for (int e = 0; e < V; ++e) six[i][e + 1] = in ? own[e] : 0.f;
      float l = __shfl_up(six[i][V], 1, kWave), r = __shfl_down(six[i][1], 1, kWave);
      if (q.first) l = (EDGE && in && q.left_off != 0) ? load_one(&el[u][i]) : 0.f;
      if (q.last) r = (EDGE && in && q.right_off != 0) ? load_one(&er[u][i]) : 0.f;
      six[i][0] = l;
      six[i][V + 1] = r;
    }
    float tile[R][V];
#pragma unroll
    for (int o = 0; o < R; ++o) {
#pragma unroll
      for (int e = 0; e < V; ++e) tile[o][e] = 0.f;
#pragma unroll
      for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
          for (int e = 0; e < V; ++e) tile[o][e] = fmaf(k[i * 3 + j], six[o + i][e + j], tile[o][e]);
    }
    fwd_levels<D, V, 1>(tile, p, sink);
    after(sink);
  };
  load_tile(0, 0);
  auto round = [&](int c) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      load_tile(u ^ 1, c + u + 1);
      __builtin_amdgcn_sched_barrier(0);  // the loads go out before the arithmetic, not after
      transform(u, c + u);
    }
  };
  int c = 0;
  if constexpr (PEEL) {
    if (1 < n_ch) {
      round(0);
      c = 2;
    }
  }
  for (; c + 1 < n_ch; c += 2) round(c);
  if (c < n_ch) transform(0, c);
}

// LDS traffic of one wave with itself: the hardware runs a wave's LDS instructions in order;
// this keeps the compiler from moving them across
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS accesses only: loads from global memory that are still in
// flight (a prefetch for a later iteration) stay in flight across it, where __syncthreads()
// would wait for them.
__device__ __forceinline__ void workgroup_lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// A wave covers (64 / lpr) strips x (lpr lanes of V columns).  lpr is the power of two that
// leaves the fewest lanes idle (ties: the wider one, for longer contiguous row segments);
// rows narrower than 16 lanes are not split further.
inline StripMap make_map(const wcc_desc &d, int V) {
  StripMap m;
  m.lanes_w = d.W / V;
  m.strips = d.H >> d.levels;
  int top = 1, lg_top = 0;
  while (top < m.lanes_w && top < kWave) { top *= 2; ++lg_top; }
  int best = top, best_lg = lg_top;
  int64_t best_units = 0;
  for (int lpr = top, lg = lg_top; lpr >= 16 || lpr == top; lpr /= 2, --lg) {
    const int spw = kWave / lpr;
    const int64_t units = (int64_t)((m.strips + spw - 1) / spw) * ((m.lanes_w + lpr - 1) / lpr);
    if (best_units == 0 || units < best_units) { best = lpr; best_lg = lg; best_units = units; }
    if (lpr == 1) break;
  }
  m.lpr = best;
  m.log_lpr = best_lg;
  m.col_segs = (m.lanes_w + best - 1) / best;
  const int spw = kWave / best;
  m.units = ((m.strips + spw - 1) / spw) * m.col_segs;
  return m;
}

// How a pass over the channels is cut into waves.
struct Plan {
  int G;       // channel groups (grid.y)
  bool split;  // forward/norm pass only: the 4 waves of a workgroup split a group's channels
  bool stream; // x is read with streaming loads (maps far larger than the memory-side cache)
};

// does a wave row span less than the plane's width (so that its end lanes have neighbours
// in memory)?
inline bool dw_needs_edges(const StripMap &m) { return m.col_segs > 1 || m.lpr < m.lanes_w; }

// Channel groups: split the channels until the launch has `want_waves` waves to cover the
// memory latency of 256 CUs, but keep at least `min_ch` channels in a group.
inline int groups_for(const wcc_desc &d, int C, int64_t want_waves, int min_ch) {
  const int V = (d.W % 4 == 0) ? 4 : 2;
  const StripMap m = make_map(d, V);
  const int64_t waves = (int64_t)m.units * d.B;
  int G = 1;
  if (waves >= want_waves / 2) return G;  // already enough strips: keep the channel walk whole
  while (waves * G < want_waves && C / (G * 2) >= min_ch) G *= 2;
  return G;
}

// The memory-side cache holds 256 MB.  An input that fits is read by the second transform pass
// from there, so it is loaded the ordinary way; one that does not is streamed past the cache.
inline bool streams(const wcc_desc &d) {
  const int64_t bytes = (int64_t)d.B * d.C_in * d.H * d.W * (d.act_dtype == WCC_BF16 ? 2 : 4);
  return bytes > ((int64_t)256 << 20);
}

// With K_dw folded in and bf16 feature maps the passes are bound by their arithmetic, not by
// bytes: there four times the waves pay (measured on the block: norm pass 300 -> 227 us, keep
// pass 492 -> 378 us), where with fp32 maps they cost 3-5 %.
inline bool arithmetic_bound(const wcc_desc &d, bool folded_dw) { return folded_dw && d.act_dtype == WCC_BF16; }

}  // namespace
}  // namespace wcc
