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

// ---- analysis ---------------------------------------------------------------------------
// STORE = false: only the |coefficient| sums are kept (the norm-only pass of the fused layer).
// SQ: the sums are of squared coefficients (one fused multiply-add each) instead.
template <int D, int V, bool STORE, bool SQ = false>
struct FwdSink {
  float *plane;  // wavelet vector of the current (b, c)
  float acc[slot_count(D, V)];
  template <int L, int J>
  __device__ __forceinline__ void put_row(const LanePos<D> &p, int i, const float (&v)[cols_at(V, L)],
                                          bool owner) {
    constexpr int CV = cols_at(V, L);
    constexpr int base = slot_base(D, V, L, J);
#pragma unroll
    for (int e = 0; e < CV; ++e) {
      float &a = acc[base + i * CV + e];
      a = SQ ? fmaf(v[e], v[e], a) : a + fabsf(v[e]);
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
__device__ __forceinline__ uint32_t to_bf16(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
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
  const uint32_t a = to_bf16(src[0]) | (to_bf16(src[1]) << 16);
  if constexpr (V == 4) {
    const uint32_t b = to_bf16(src[2]) | (to_bf16(src[3]) << 16);
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
  const uint32_t a = to_bf16(src[0]) | (to_bf16(src[1]) << 16);
  if constexpr (V == 4) {
    stream_u2 t;
    t.x = a;
    t.y = to_bf16(src[2]) | (to_bf16(src[3]) << 16);
    __builtin_nontemporal_store(t, reinterpret_cast<stream_u2 *>(dst));
  } else {
    __builtin_nontemporal_store(a, reinterpret_cast<uint32_t *>(dst));
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

// x [B, C, H, W] -> coef [B, C, N]; partial norms over this block's channel group to
// norm_part [G, B, N] (nullable).  block = 256.
// SPLIT = false: grid = (ceil(units/4), G, B); each wave of a workgroup takes its own strip unit
//                and walks all channels of the group.
// SPLIT = true:  grid = (units, G, B); the four waves share one strip unit and take a quarter
//                of the group's channels each (four times the waves in flight for the same
//                number of partial-norm planes); their |coefficient| sums meet in LDS and are
//                added in wave order.
// DWM: 0 = x is transformed as it is; 1, 2 = K_dw x is (wdw [C, 3, 3]; 2: the outside columns
// of a wave row's first and last lane exist and are read).
// XT: float or bf16_t, the storage type of x.  SQ: sums of squares instead of absolute values.
template <int D, int V, bool SPLIT, bool STORE, int PF, int DWM, class XT, bool SQ = false,
          bool NT = false>
__global__ __launch_bounds__(256) void haar_fwd_kernel(const XT *__restrict__ x,
                                                       float *__restrict__ coef,
                                                       float *__restrict__ norm_part, Geo g,
                                                       StripMap m, int C, int Cg, int B,
                                                       SelectPrep prep,
                                                       const float *__restrict__ wdw) {
  constexpr int NS = slot_count(D, V);
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int unit = SPLIT ? (int)blockIdx.x : (int)blockIdx.x * 4 + wv;
  const int grp = blockIdx.y, b = blockIdx.z;
  // one workgroup per sample clears the state of the selection that follows this kernel
  if (blockIdx.x == 0 && grp == 0) prep_sample(prep, b, threadIdx.x, 256);
  LanePos<D> p;
  int row0, col0;
  locate<D, V>(m, g, unit, p, row0, col0);
  (void)coef;
  int c0 = grp * Cg, c1 = min(C, c0 + Cg);
  if constexpr (SPLIT) {
    const int Cw = (c1 - c0 + 3) / 4;
    c0 = c0 + wv * Cw;
    c1 = min(c1, c0 + Cw);
  }

  FwdSink<D, V, STORE, SQ> sink;
#pragma unroll
  for (int s = 0; s < NS; ++s) sink.acc[s] = 0.f;

  if (p.active && c0 < c1) {
    const XT *src = x + ((size_t)b * C + c0) * g.N + (size_t)row0 * g.W + col0;
    sink.plane = STORE ? coef + ((size_t)b * C + c0) * g.N : nullptr;
    const int64_t N = g.N;
    if constexpr (DWM == 0) {
      channel_loop<D, V, PF, NT>(src, N, g.W, c1 - c0, p, sink, [N](FwdSink<D, V, STORE, SQ> &sk) {
        if (STORE) sk.plane += N;
      });
    } else {
      const DwLane q = dw_lane<D, V>(g, m, p, row0, col0);
      channel_loop_dw<D, V, DWM == 2, false, NT>(src, wdw + (size_t)c0 * 9, N, c1 - c0, q, p, sink,
                                             [](FwdSink<D, V, STORE, SQ> &) {});
    }
  }

  if (norm_part == nullptr) return;
  if constexpr (SPLIT) {
    __shared__ float comb[3][NS][kWave];
    if (wv > 0) {
#pragma unroll
      for (int s = 0; s < NS; ++s) comb[wv - 1][s][lane] = sink.acc[s];
    }
    __syncthreads();
    if (wv > 0) return;
#pragma unroll
    for (int s = 0; s < NS; ++s)
      sink.acc[s] = ((sink.acc[s] + comb[0][s][lane]) + comb[1][s][lane]) + comb[2][s][lane];
  }
  if (!p.active) return;
  float *np = norm_part + ((size_t)grp * B + b) * g.N;
  // write the accumulated |coefficient| sums with the same addressing as the coefficients
  auto flush = [&](auto Lc, auto Jc) {
    constexpr int L = decltype(Lc)::value, J = decltype(Jc)::value;
    constexpr int CV = cols_at(V, L), S2 = span_at(V, L);
    const bool owner = (S2 == 1) || ((p.lc & (S2 - 1)) == 0);
    if (!owner) return;
#pragma unroll
    for (int i = 0; i < rows_at(D, L); ++i) {
      float *dst = np + (J * p.nl[L] + p.off[L] + i * p.rowlen[L]);
      if constexpr (CV == 2) {
        *reinterpret_cast<float2 *>(dst) = make_float2(sink.acc[slot_base(D, V, L, J) + i * CV],
                                                       sink.acc[slot_base(D, V, L, J) + i * CV + 1]);
      } else {
#pragma unroll
        for (int e = 0; e < CV; ++e) dst[e] = sink.acc[slot_base(D, V, L, J) + i * CV + e];
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

// LDS traffic of one wave with itself: the hardware runs a wave's LDS instructions in order;
// this keeps the compiler from moving them across
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- second pass of the fused layer: transform again, keep only the selected positions ----
// xc[b, c, jmap[b, q]] = HWT_d(x[b, c])[q] for the kept q; dropped coefficients never reach
// memory.  Also raises the alpha slots to max |kept coefficient| (nullable).
// Q8: the clipping parameter is known beforehand (the caller supplied it), so the kept
// coefficients leave the chip as signed 8-bit codes (Eq. quantweights) instead of fp32.
template <int D, int V, bool Q8>
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
#pragma unroll
    for (int e = 0; e < CV; ++e) {
      const int s = base + i * CV + e;
      if constexpr (Q8) {
        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(int8_t)quant.code(v[e]), xc_c, at[s], 0, 0);
      } else {
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
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const float v = __uint_as_float(tile[cell[i]]);
      if constexpr (Q8) {
        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(int8_t)quant.code(v), xc_c, at[i], 0, 0);
      } else {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), xc_c, at[i], 0, 0);
        vmax = fmaxf(vmax, at[i] != kDropped ? fabsf(v) : 0.f);
      }
    }
    wave_lds_fence();
  }
};

// grid = (ceil(units/4), G, B), block = 256.  DWM as in haar_fwd_kernel.  Q8: xc is int8 codes
// for the clipping parameter q_alpha (> 0), and alpha_slots must be null.
template <int D, int V, int PF, int DWM, bool Q8, class XT, bool NT = false>
__global__ __launch_bounds__(256) void haar_keep_kernel(const XT *__restrict__ x,
                                                        const int32_t *__restrict__ jmap,
                                                        void *__restrict__ xc, float *alpha_slots,
                                                        Geo g, StripMap m, int C, int Cg, int64_t k,
                                                        const float *__restrict__ wdw,
                                                        float q_alpha) {
  __shared__ float wmax[4];
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int grp = blockIdx.y, b = blockIdx.z;
  LanePos<D> p;
  int row0, col0;
  const bool active = locate<D, V>(m, g, unit, p, row0, col0);
  const int c0 = grp * Cg, c1 = min(C, c0 + Cg);

  using Sink = KeepSink<D, V, Q8>;
  Sink sink(Q8 ? q_alpha : 0.f);
  const int32_t *jm = jmap + (size_t)b * g.N;
  auto fetch = [&](auto Lc, auto Jc) {
    constexpr int L = decltype(Lc)::value, J = decltype(Jc)::value;
    constexpr int CV = cols_at(V, L), S2 = span_at(V, L);
    const bool owner = (S2 == 1) || ((p.lc & (S2 - 1)) == 0);
#pragma unroll
    for (int i = 0; i < rows_at(D, L); ++i)
#pragma unroll
      for (int e = 0; e < CV; ++e) {
        constexpr int base = slot_base(D, V, L, J);
        const int s = base + i * CV + e;
        int j = -1;
        if (active && owner) j = jm[J * p.nl[L] + p.off[L] + i * p.rowlen[L] + e];
        sink.at[s] = (uint32_t)j;  // (turned into a byte offset below, once all loads are out)
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
  using Out = typename Sink::Out;
  const XT *src = x + ((size_t)b * C + c0) * g.N + (size_t)row0 * g.W + col0;
  Out *plane = static_cast<Out *>(xc) + ((size_t)b * C + c0) * k;
  // walks the group's channels with whichever sink; returns its max |kept coefficient|
  auto walk = [&](auto &sk, auto &&next_channel) {
    sk.vmax = 0.f;
    sk.aim(plane, k);
    if constexpr (DWM == 0) {
      channel_loop<D, V, PF, NT>(src, g.N, g.W, c1 - c0, p, sk, next_channel);
    } else {
      const DwLane q = dw_lane<D, V>(g, m, p, row0, col0);
      channel_loop_dw<D, V, DWM == 2, true, false>(src, wdw + (size_t)c0 * 9, g.N, c1 - c0, q, p, sk,
                                                   next_channel);
    }
    return sk.vmax;
  };

  float mx = 0.f;
  bool done = false;
  // Dense stores pay where a strip keeps at most half of its slots' worth of positions.  (With
  // K_dw folded in the kernel is bound by its arithmetic and registers; there the staging
  // measured 5-10 % slower than one store per slot.)
  constexpr int NS = slot_count(D, V);
  constexpr bool kStaged = V == 4 && (D == 2 || D == 3) && DWM == 0;
  if constexpr (kStaged) {
    __shared__ uint32_t tiles[4][NS * kWave];
    constexpr int kRankBits = 20;  // list entry = rank | tile index << 20
    int count = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) count += __popcll(__ballot((int)sink.at[s] >= 0));
    const int ni = (count + kWave - 1) / kWave;
    const bool whole = __ballot(active) == ~(uint64_t)0;  // (a ragged wave takes the plain path)
    if (whole && c0 < c1 && ni <= NS / 2 && ni <= 16 && k <= ((int64_t)1 << kRankBits)) {
      const int lane = threadIdx.x & (kWave - 1);
      uint32_t *tile = tiles[threadIdx.x >> 6];
      // pack (rank, tile index): slot-major, then lane (a band row's kept positions have
      // consecutive ranks).  The tile is scratch for the list before it becomes the staging area.
      int running = 0;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const int j = (int)sink.at[s];
        const uint64_t kept = __ballot(j >= 0);
        const int to = running + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(kept >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)kept, 0u));
        if (j >= 0) tile[to] = (uint32_t)j | ((uint32_t)(s * kWave + lane) << kRankBits);
        running += __popcll(kept);
      }
      wave_lds_fence();
      auto run = [&](auto ni_c) {
        constexpr int NI = decltype(ni_c)::value;
        KeepStagedSink<D, V, Q8, NI> st(Q8 ? q_alpha : 0.f);
        st.tile = tile;
        st.lane = lane;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          const int e = lane + kWave * i;
          const uint32_t packed = e < count ? tile[e] : 0u;
          st.cell[i] = e < count ? packed >> kRankBits : (uint32_t)lane;
          st.at[i] = e < count ? (packed & ((1u << kRankBits) - 1u)) * (uint32_t)sizeof(Out) : Sink::kDropped;
        }
        wave_lds_fence();
        mx = walk(st, [&plane, k](auto &sk) {
          sk.flush();
          plane += k;
          sk.aim(plane, k);
        });
      };
      if (ni <= 4) run(std::integral_constant<int, 4>{});
      else if (ni <= 8) run(std::integral_constant<int, 8>{});
      else run(std::integral_constant<int, 16>{});  // (ni <= 16 is part of the condition above)
      done = true;
    }
  }
  if (!done && active && c0 < c1) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
      sink.at[s] = (int)sink.at[s] >= 0 ? sink.at[s] * (uint32_t)sizeof(Out) : Sink::kDropped;
    mx = walk(sink, [&plane, k](Sink &sk) {
      plane += k;
      sk.aim(plane, k);
    });
  }
  if (alpha_slots == nullptr) return;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    // integer max on the bit pattern of a non-negative float: exact and order-independent;
    // workgroups spread over the slots because atomics on one address serialise
    unsigned int *a = reinterpret_cast<unsigned int *>(alpha_slots) +
                      ((blockIdx.x + 3u * blockIdx.y + 11u * blockIdx.z) & (kAlphaSlots - 1));
    const unsigned int mine = __float_as_uint(mx);
    if (mine > __hip_atomic_load(a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(a, mine);
  }
}

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
// LDS tile laid out [slot][lane] whose other cells stay zero, and every lane reads its slots
// back from there.  Lanes outside the plane take part in the list work and send their stores
// to a scratch line.  Strips that keep more than kInvCap positions, layers with more than 2^20
// kept positions, and d = 4 (whose tile would not fit) take the plain path: ranks in registers,
// one conditional load per slot.
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

// The channel walk of the staged path with NI dense fetches per channel.  mine[i]: the lane's
// list entries (kInvNone: padding).  row_step: W for lanes inside the plane, 0 for the others
// (whose dst is the scratch line).
// RES: res + (what dst points at, relative to the output tensor) is added to every stored row.
template <int D, int V, int NI, bool RES, class YT>
__device__ __forceinline__ void inv_staged_walk(const float *__restrict__ plane, int64_t k, int n_ch,
                                                const uint32_t (&mine)[kInvCap / kWave],
                                                uint32_t *tile, const InvStaged<D, V> &staged,
                                                const LanePos<D> &p, YT *dst, int row_step,
                                                int64_t dst_step, const YT *res) {
  constexpr int R = 1 << D;
  constexpr uint32_t kRank = (1u << kInvRankBits) - 1u;
  float vn[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) vn[i] = plane[mine[i] == kInvNone ? 0u : (mine[i] & kRank)];
  auto channel = [&](int c) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
      if (mine[i] != kInvNone) tile[mine[i] >> kInvRankBits] = __float_as_uint(vn[i]);
    // the next channel's values travel while this one is built (past the end: the last again)
    const float *nx = plane + (size_t)min(c + 1, n_ch - 1) * k;
#pragma unroll
    for (int i = 0; i < NI; ++i) vn[i] = nx[mine[i] == kInvNone ? 0u : (mine[i] & kRank)];
    float skip[RES ? R : 1][V];
    if constexpr (RES) {
#pragma unroll
      for (int r = 0; r < R; ++r) load_row_stream<V>(res + (size_t)r * row_step, skip[r]);
    }
    __builtin_amdgcn_sched_barrier(0);
    wave_lds_fence();
    float out[R][V];
    inv_levels<D, V, 1>(out, p, staged);
    wave_lds_fence();
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (RES) {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < V; ++e) out[r][e] += skip[r][e];
      res += dst_step;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) store_row_stream<V>(dst + (size_t)r * row_step, out[r]);
    dst += dst_step;
  };
  // The first channel stands outside the loop: at the loop head the outstanding memory
  // operations are then "fetches, then R stores" on both incoming paths, and the wait for a
  // fetch need not cover the stores.
  channel(0);
  for (int c = 1; c < n_ch; ++c) channel(c);
}

// yc [B, C, k] + jmap [B, N] -> y [B, C, H, W].  grid = (ceil(units/4), G, B), block = 256.
// scratch: 1 KiB that lanes outside the plane may overwrite.  RES: y = residual + (the above),
// residual [B, C, H, W] (the skip connection of Eq. (inverted)); it may be y itself.
// YT: float or bf16_t, the storage type of y and of the residual.
template <int D, int V, bool RES, class YT>
__global__ __launch_bounds__(256) void scatter_ihaar_kernel(const float *__restrict__ yc,
                                                            const int32_t *__restrict__ jmap,
                                                            YT *y, Geo g, StripMap m, int C,
                                                            int Cg, int64_t k, float *scratch,
                                                            const YT *residual) {
  constexpr int R = 1 << D;
  constexpr int NS = slot_count(D, V);
  constexpr bool kStaged = D <= 3;  // the [slot][lane] tiles of four waves fit in LDS
  constexpr int CAP = NS * kWave < kInvCap ? NS * kWave : kInvCap;  // entries a wave can pack
  static_assert(NS <= 128, "slot mask is 128 bits wide");
  static_assert(!kStaged || NS * kWave <= (1 << (32 - kInvRankBits)), "cell index fits above the rank");
  __shared__ uint32_t tiles[kStaged ? 4 : 1][kStaged ? NS * kWave : 1];
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + wv;
  const int grp = blockIdx.y, b = blockIdx.z;
  LanePos<D> p;
  int row0, col0;
  const bool active = locate<D, V>(m, g, unit, p, row0, col0);
  const int c0 = grp * Cg, c1 = min(C, c0 + Cg);
  if (__ballot(active) == 0 || c0 >= c1) return;  // whole waves leave

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
          if (j >= 0) tile[at] = (uint32_t)j | ((uint32_t)(s * kWave + lane) << kInvRankBits);
          running += __popcll(kept);
        }
      }
      wave_lds_fence();
      uint32_t mine[kInvCap / kWave];  // this lane's share of the list: entries lane + 64 i
#pragma unroll
      for (int i = 0; i < kInvCap / kWave; ++i) {
        const int e = lane + 64 * i;
        mine[i] = (i < CAP / kWave && e < count) ? tile[e] : kInvNone;
      }
      wave_lds_fence();
#pragma unroll
      for (int s = 0; s < NS; ++s) tile[s * kWave + lane] = 0u;

      InvStaged<D, V> staged;
      staged.cell = reinterpret_cast<const float *>(tile) + lane;
      staged.any[0] = src.any[0];
      staged.any[1] = src.any[1];
      YT *sink_line = reinterpret_cast<YT *>(scratch) + lane * V;
      YT *to = active ? dst : sink_line;
      const YT *res = (RES && active) ? residual + first : sink_line;
      const int row_step = active ? g.W : 0;
      const int64_t dst_step = active ? g.N : 0;
      const int ni = (count + 63) >> 6;
      if (ni <= 4)
        inv_staged_walk<D, V, 4, RES, YT>(plane, k, c1 - c0, mine, tile, staged, p, to, row_step, dst_step, res);
      else if (ni <= 8)
        inv_staged_walk<D, V, 8, RES, YT>(plane, k, c1 - c0, mine, tile, staged, p, to, row_step, dst_step, res);
      else
        inv_staged_walk<D, V, 16, RES, YT>(plane, k, c1 - c0, mine, tile, staged, p, to, row_step, dst_step, res);
      return;
    }
  }

  // plain path
  if (!active) return;
  src.plane = plane;
  const YT *res = RES ? residual + first : nullptr;
  for (int c = c0; c < c1; ++c) {
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
      res += g.N;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) store_row_stream<V>(dst + (size_t)r * g.W, out[r]);
    src.plane += k;
    dst += g.N;
  }
}

// ---- small helpers ----------------------------------------------------------------------------
// norm[i] = sum_g part[g][i], groups added in increasing order (fixed order: reproducible).
__global__ __launch_bounds__(256) void norm_reduce_kernel(const float *__restrict__ part, int G,
                                                          int64_t BN4, float4 *__restrict__ norm) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= BN4) return;
  const float4 *p = reinterpret_cast<const float4 *>(part);
  float4 s = p[i];
  for (int gi = 1; gi < G; ++gi) {
    const float4 t = p[(int64_t)gi * BN4 + i];
    s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
  }
  norm[i] = s;
}

// norm[b, q] = sum_c |coef[b, c, q]| (SQ: sum_c coef^2), channels in increasing order.
// grid = (ceil(N/4/256), B)
template <bool SQ>
__global__ __launch_bounds__(256) void channel_norm_kernel(const float *__restrict__ coef, int C,
                                                           int64_t N, float *__restrict__ norm) {
  const int64_t i4 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (i4 * 4 >= N) return;
  const float4 *p = reinterpret_cast<const float4 *>(coef + (size_t)b * C * N) + i4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c = 0; c < C; ++c) {
    const float4 t = p[(size_t)c * (N / 4)];
    if constexpr (SQ) {
      s.x = fmaf(t.x, t.x, s.x); s.y = fmaf(t.y, t.y, s.y);
      s.z = fmaf(t.z, t.z, s.z); s.w = fmaf(t.w, t.w, s.w);
    } else {
      s.x += fabsf(t.x); s.y += fabsf(t.y); s.z += fabsf(t.z); s.w += fabsf(t.w);
    }
  }
  reinterpret_cast<float4 *>(norm + (size_t)b * N)[i4] = s;
}

// A wave covers (64 / lpr) strips x (lpr lanes of V columns).  lpr is the power of two that
// leaves the fewest lanes idle (ties: the wider one, for longer contiguous row segments);
// rows narrower than 16 lanes are not split further.
StripMap make_map(const wcc_desc &d, int V) {
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

// x is fp32, or bf16 when the layer's activations are stored that way (fused calls only)
template <int D, int V, bool STORE>
hipError_t fwd_launch(const wcc_desc &d, const void *x, float *coef, float *norm_part, Plan pl,
                      const SelectPrep &prep, const float *wdw, hipStream_t s);

// does a wave row span less than the plane's width (so that its end lanes have neighbours
// in memory)?
bool dw_needs_edges(const StripMap &m) { return m.col_segs > 1 || m.lpr < m.lanes_w; }

template <int D, int V, bool STORE, class XT>
hipError_t fwd_launch_t(const wcc_desc &d, const XT *x, float *coef, float *norm_part, Plan pl,
                        const SelectPrep &prep, const float *wdw, hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = make_map(d, V);
  const int Cg = (d.C_in + pl.G - 1) / pl.G;
  const dim3 grid_split(m.units, pl.G, d.B), grid_flat((m.units + 3) / 4, pl.G, d.B), block(256);
#define WCC_FWD(SPLIT, PF, DWM)                                                                       \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, SPLIT, STORE, PF, DWM, XT>),                              \
                     SPLIT ? grid_split : grid_flat, block, 0, s, x, coef, norm_part, g, m, d.C_in,   \
                     Cg, d.B, prep, wdw)
  if (d.norm == WCC_NORM_L2) {
    // sums of squares: the norm-only pass over fp32 maps, prefetch depth 1
    if constexpr (!STORE && std::is_same<XT, float>::value) {
#define WCC_FWD_SQ(SPLIT, DWM)                                                                        \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, SPLIT, false, 1, DWM, float, true>),                      \
                     SPLIT ? grid_split : grid_flat, block, 0, s, x, coef, norm_part, g, m, d.C_in,   \
                     Cg, d.B, prep, wdw)
#define WCC_FWD_SQ_NT(DWM)                                                                            \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, false, false, 1, DWM, float, true, true>), grid_flat,     \
                     block, 0, s, x, coef, norm_part, g, m, d.C_in, Cg, d.B, prep, wdw)
      const bool nt = pl.stream && !pl.split;  // (an input far larger than the memory-side cache)
      if (wdw != nullptr) {
        if constexpr (V == 4) {
          const bool edges = dw_needs_edges(m);
          if (nt)            { if (edges) WCC_FWD_SQ_NT(2); else WCC_FWD_SQ_NT(1); }
          else if (pl.split) { if (edges) WCC_FWD_SQ(true, 2); else WCC_FWD_SQ(true, 1); }
          else               { if (edges) WCC_FWD_SQ(false, 2); else WCC_FWD_SQ(false, 1); }
          return hipGetLastError();
        }
        return hipErrorInvalidValue;
      }
      if (nt) WCC_FWD_SQ_NT(0); else if (pl.split) WCC_FWD_SQ(true, 0); else WCC_FWD_SQ(false, 0);
#undef WCC_FWD_SQ_NT
#undef WCC_FWD_SQ
      return hipGetLastError();
    }
    return hipErrorInvalidValue;
  }
  if constexpr (!STORE) {
    if (pl.stream && !pl.split) {  // an input far larger than the memory-side cache, read once
#define WCC_FWD_NT(DWM)                                                                               \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, false, false, 1, DWM, XT, false, true>), grid_flat,       \
                     block, 0, s, x, coef, norm_part, g, m, d.C_in, Cg, d.B, prep, wdw)
      if (wdw != nullptr) {
        if constexpr (V == 4) {
          if (dw_needs_edges(m)) WCC_FWD_NT(2); else WCC_FWD_NT(1);
          return hipGetLastError();
        }
        return hipErrorInvalidValue;
      }
      WCC_FWD_NT(0);
#undef WCC_FWD_NT
      return hipGetLastError();
    }
  }
  if constexpr (!STORE && V == 4) {
    if (wdw != nullptr) {  // K_dw in front of the transform (norm-only pass)
      const bool edges = dw_needs_edges(m);
      if (pl.split) { if (edges) WCC_FWD(true, 1, 2); else WCC_FWD(true, 1, 1); }
      else          { if (edges) WCC_FWD(false, 1, 2); else WCC_FWD(false, 1, 1); }
      return hipGetLastError();
    }
  }
  if (wdw != nullptr) return hipErrorInvalidValue;
  // (a prefetch depth of two channels was measured on every workload and never paid)
  if (pl.split) WCC_FWD(true, 1, 0); else WCC_FWD(false, 1, 0);
#undef WCC_FWD
  return hipGetLastError();
}

template <int D, int V, bool STORE>
hipError_t fwd_launch(const wcc_desc &d, const void *x, float *coef, float *norm_part, Plan pl,
                      const SelectPrep &prep, const float *wdw, hipStream_t s) {
  if constexpr (!STORE) {
    if (d.act_dtype == WCC_BF16)
      return fwd_launch_t<D, V, STORE>(d, static_cast<const bf16_t *>(x), coef, norm_part, pl, prep, wdw, s);
  }
  return fwd_launch_t<D, V, STORE>(d, static_cast<const float *>(x), coef, norm_part, pl, prep, wdw, s);
}

template <int D, int V, class XT>
hipError_t keep_launch_t(const wcc_desc &d, int64_t k, const XT *x, const int32_t *jmap, void *xc,
                         float *alpha_slots, Plan pl, const float *wdw, float q_alpha, hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = make_map(d, V);
  const int Cg = (d.C_in + pl.G - 1) / pl.G;
  dim3 grid((m.units + 3) / 4, pl.G, d.B);
  const bool q8 = q_alpha > 0.f;
#define WCC_KEEP(PF, DWM)                                                                          \
  do {                                                                                             \
    if (q8)                                                                                        \
      hipLaunchKernelGGL((haar_keep_kernel<D, V, PF, DWM, true, XT>), grid, dim3(256), 0, s, x,   \
                         jmap, xc, nullptr, g, m, d.C_in, Cg, k, wdw, q_alpha);                    \
    else                                                                                           \
      hipLaunchKernelGGL((haar_keep_kernel<D, V, PF, DWM, false, XT>), grid, dim3(256), 0, s, x,  \
                         jmap, xc, alpha_slots, g, m, d.C_in, Cg, k, wdw, 0.f);                    \
  } while (0)
  if constexpr (V == 4) {
    if (wdw != nullptr) {  // K_dw in front of the transform
      if (dw_needs_edges(m)) WCC_KEEP(1, 2); else WCC_KEEP(1, 1);
      return hipGetLastError();
    }
  }
  if (wdw != nullptr) return hipErrorInvalidValue;
  if (pl.stream) {
    if (q8)
      hipLaunchKernelGGL((haar_keep_kernel<D, V, 1, 0, true, XT, true>), grid, dim3(256), 0, s, x,
                         jmap, xc, nullptr, g, m, d.C_in, Cg, k, wdw, q_alpha);
    else
      hipLaunchKernelGGL((haar_keep_kernel<D, V, 1, 0, false, XT, true>), grid, dim3(256), 0, s, x,
                         jmap, xc, alpha_slots, g, m, d.C_in, Cg, k, wdw, 0.f);
    return hipGetLastError();
  }
  WCC_KEEP(1, 0);
#undef WCC_KEEP
  return hipGetLastError();
}

template <int D, int V>
hipError_t keep_launch(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap, void *xc,
                       float *alpha_slots, Plan pl, const float *wdw, float q_alpha, hipStream_t s) {
  if (d.act_dtype == WCC_BF16)
    return keep_launch_t<D, V>(d, k, static_cast<const bf16_t *>(x), jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
  return keep_launch_t<D, V>(d, k, static_cast<const float *>(x), jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
}

template <int D, int V>
hipError_t inv_launch(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap, void *y,
                      int G, float *scratch, const void *residual, hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = make_map(d, V);
  const int Cg = (d.C_out + G - 1) / G;
  dim3 grid((m.units + 3) / 4, G, d.B);
#define WCC_INV(RES, YT)                                                                          \
  hipLaunchKernelGGL((scatter_ihaar_kernel<D, V, RES, YT>), grid, dim3(256), 0, s, yc, jmap,      \
                     static_cast<YT *>(y), g, m, d.C_out, Cg, k, scratch,                         \
                     static_cast<const YT *>(residual))
  if (d.act_dtype == WCC_BF16) { if (residual) WCC_INV(true, bf16_t); else WCC_INV(false, bf16_t); }
  else                         { if (residual) WCC_INV(true, float); else WCC_INV(false, float); }
#undef WCC_INV
  return hipGetLastError();
}

// Channel groups: split the channels until the launch has `want_waves` waves to cover the
// memory latency of 256 CUs, but keep at least `min_ch` channels in a group.
int groups_for(const wcc_desc &d, int C, int64_t want_waves, int min_ch) {
  const int V = (d.W % 4 == 0) ? 4 : 2;
  const StripMap m = make_map(d, V);
  const int64_t waves = (int64_t)m.units * d.B;
  int G = 1;
  if (waves >= want_waves / 2) return G;  // already enough strips: keep the channel walk whole
  while (waves * G < want_waves && C / (G * 2) >= min_ch) G *= 2;
  return G;
}

}  // namespace

// Every forward group costs one partial-norm plane (written once, read once): with >= 16
// channels a group that is at most 1/16 of the transform's own traffic.  Measured on gfx950:
// about a thousand waves, each walking as many channels as possible, stream best; more
// groups only pay when a layer has fewer strips than that.
//
// With K_dw folded in and bf16 feature maps the passes are bound by their arithmetic, not by
// bytes: there four times the waves pay (measured on the block: norm pass 300 -> 227 us, keep
// pass 492 -> 378 us), where with fp32 maps they cost 3-5 %.
bool arithmetic_bound(const wcc_desc &d, bool folded_dw) { return folded_dw && d.act_dtype == WCC_BF16; }

int forward_groups(const wcc_desc &d, bool folded_dw) {
  return groups_for(d, d.C_in, arithmetic_bound(d, folded_dw) ? 4096 : 1024, 16);
}

template <bool STORE>
hipError_t fwd_dispatch(const wcc_desc &d, const void *x, float *coef, float *norm_part, Plan pl,
                        const SelectPrep &prep, const float *wdw, hipStream_t s) {
  const bool v4 = d.W % 4 == 0;
  switch (d.levels) {
    case 1: return v4 ? fwd_launch<1, 4, STORE>(d, x, coef, norm_part, pl, prep, wdw, s)
                      : fwd_launch<1, 2, STORE>(d, x, coef, norm_part, pl, prep, wdw, s);
    case 2: return fwd_launch<2, 4, STORE>(d, x, coef, norm_part, pl, prep, wdw, s);
    case 3: return fwd_launch<3, 4, STORE>(d, x, coef, norm_part, pl, prep, wdw, s);
    case 4: return fwd_launch<4, 4, STORE>(d, x, coef, norm_part, pl, prep, wdw, s);
  }
  return hipErrorInvalidValue;
}

hipError_t keep_dispatch(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap, void *xc,
                         float *alpha_slots, Plan pl, const float *wdw, float q_alpha, hipStream_t s) {
  const bool v4 = d.W % 4 == 0;
  switch (d.levels) {
    case 1: return v4 ? keep_launch<1, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, s)
                      : keep_launch<1, 2>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
    case 2: return keep_launch<2, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
    case 3: return keep_launch<3, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
    case 4: return keep_launch<4, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
  }
  return hipErrorInvalidValue;
}

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

// G is fixed by the workspace layout (one partial-norm plane per group).  On small layers,
// where even the groups leave fewer than 1024 waves, the four waves of a workgroup split a
// group's channels (if each still gets >= 2).
// The memory-side cache holds 256 MB.  An input that fits is read by the second transform pass
// from there, so it is loaded the ordinary way; one that does not is streamed past the cache.
bool streams(const wcc_desc &d) {
  const int64_t bytes = (int64_t)d.B * d.C_in * d.H * d.W * (d.act_dtype == WCC_BF16 ? 2 : 4);
  return bytes > ((int64_t)256 << 20);
}

Plan fwd_plan(const wcc_desc &d, int G) {
  const int Cg = (d.C_in + G - 1) / G;
  const StripMap m = make_map(d, (d.W % 4 == 0) ? 4 : 2);
  const int64_t waves = (int64_t)m.units * d.B * G;
  return Plan{G, waves < 1024 && Cg >= 8, streams(d)};
}

hipError_t launch_haar_fwd(const wcc_desc &d, const float *x, float *coef, float *norm_part, int G,
                           const SelectPrep &prep, hipStream_t s) {
  return fwd_dispatch<true>(d, x, coef, norm_part, fwd_plan(d, G), prep, nullptr, s);
}

hipError_t launch_haar_norm(const wcc_desc &d, const void *x, float *norm_part, int G,
                            const SelectPrep &prep, const float *wdw, hipStream_t s) {
  const Plan pl = fwd_plan(d, G);
  return fwd_dispatch<false>(d, x, nullptr, norm_part, pl, prep, wdw, s);
}

hipError_t launch_haar_keep(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap,
                            void *xc, float *alpha_slots, const float *wdw, float q_alpha,
                            hipStream_t s) {
  const Plan pl{groups_for(d, d.C_in, arithmetic_bound(d, wdw != nullptr) ? 4096 : 1024, 8), false,
                streams(d)};
  return keep_dispatch(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, s);
}

hipError_t launch_scatter_ihaar(const wcc_desc &d, int64_t k, const float *yc, const int32_t *jmap,
                                void *y, float *scratch, const void *residual, hipStream_t s) {
  return inv_dispatch(d, k, yc, jmap, y, groups_for(d, d.C_out, 2048, 8), scratch, residual, s);
}

hipError_t launch_norm_reduce(const float *norm_part, int G, int64_t BN, float *norm, hipStream_t s) {
  const int64_t n4 = BN / 4;
  hipLaunchKernelGGL(norm_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                     norm_part, G, n4, reinterpret_cast<float4 *>(norm));
  return hipGetLastError();
}

hipError_t launch_channel_norm(const float *coef, int B, int C, int64_t N, bool squares,
                               float *norm, hipStream_t s) {
  dim3 grid((unsigned)((N / 4 + 255) / 256), B);
  if (squares)
    hipLaunchKernelGGL(channel_norm_kernel<true>, grid, dim3(256), 0, s, coef, C, N, norm);
  else
    hipLaunchKernelGGL(channel_norm_kernel<false>, grid, dim3(256), 0, s, coef, C, N, norm);
  return hipGetLastError();
}

}  // namespace wcc
