// First transform pass of the fused layer and the stand-alone analysis (Eq. HaarKernel,
// Eq. wavelet_transform), with the channel norm of Alg. 1 fused in.
#include "strip_io.h"

namespace wcc {
namespace {

// x [B, C, H, W] -> coef [B, C, N]; partial norms over this block's channel group to
// norm_part [G, B, N] (nullable); without STORE also the group's max |coefficient| per position
// to max_part [G, B, N] (nullable).  block = 256.
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
                                                       float *__restrict__ norm_part,
                                                       float *__restrict__ max_part, Geo g,
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
  constexpr bool MX = FwdSink<D, V, STORE, SQ>::MX;
  if constexpr (MX) {
#pragma unroll
    for (int s = 0; s < NS; ++s) sink.top[s] = 0.f;
  }

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
    if (wv == 0) {
#pragma unroll
      for (int s = 0; s < NS; ++s)
        sink.acc[s] = ((sink.acc[s] + comb[0][s][lane]) + comb[1][s][lane]) + comb[2][s][lane];
    }
    if constexpr (MX) {
      if (max_part != nullptr) {  // (uniform over the grid) the maxima meet in the same buffer
        __syncthreads();
        if (wv > 0) {
#pragma unroll
          for (int s = 0; s < NS; ++s) comb[wv - 1][s][lane] = sink.top[s];
        }
        __syncthreads();
        if (wv == 0) {
#pragma unroll
          for (int s = 0; s < NS; ++s)
            sink.top[s] = fmaxf(fmaxf(sink.top[s], comb[0][s][lane]), fmaxf(comb[1][s][lane], comb[2][s][lane]));
        }
      }
    }
    if (wv > 0) return;
  }
  if (!p.active) return;
  write_slots<D, V>(norm_part + ((size_t)grp * B + b) * g.N, sink.acc, p);
  if constexpr (MX) {
    if (max_part != nullptr) write_slots<D, V>(max_part + ((size_t)grp * B + b) * g.N, sink.top, p);
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

// x is fp32, or bf16 when the layer's activations are stored that way (fused calls only)
template <int D, int V, bool STORE>
hipError_t fwd_launch(const wcc_desc &d, const void *x, float *coef, float *norm_part,
                      float *max_part, Plan pl, const SelectPrep &prep, const float *wdw, hipStream_t s);

template <int D, int V, bool STORE, class XT>
hipError_t fwd_launch_t(const wcc_desc &d, const XT *x, float *coef, float *norm_part,
                        float *max_part, Plan pl, const SelectPrep &prep, const float *wdw,
                        hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = make_map(d, V);
  const int Cg = (d.C_in + pl.G - 1) / pl.G;
  const dim3 grid_split(m.units, pl.G, d.B), grid_flat((m.units + 3) / 4, pl.G, d.B), block(256);
#define WCC_FWD(SPLIT, PF, DWM)                                                                       \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, SPLIT, STORE, PF, DWM, XT>),                              \
                     SPLIT ? grid_split : grid_flat, block, 0, s, x, coef, norm_part, max_part, g, m, d.C_in,   \
                     Cg, d.B, prep, wdw)
  if (d.norm == WCC_NORM_L2) {
    // sums of squares: the norm-only pass over fp32 maps, prefetch depth 1
    if constexpr (!STORE && std::is_same<XT, float>::value) {
#define WCC_FWD_SQ(SPLIT, DWM)                                                                        \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, SPLIT, false, 1, DWM, float, true>),                      \
                     SPLIT ? grid_split : grid_flat, block, 0, s, x, coef, norm_part, max_part, g, m, d.C_in,   \
                     Cg, d.B, prep, wdw)
#define WCC_FWD_SQ_NT(DWM)                                                                            \
  hipLaunchKernelGGL((haar_fwd_kernel<D, V, false, false, 1, DWM, float, true, true>), grid_flat,     \
                     block, 0, s, x, coef, norm_part, max_part, g, m, d.C_in, Cg, d.B, prep, wdw)
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
                     block, 0, s, x, coef, norm_part, max_part, g, m, d.C_in, Cg, d.B, prep, wdw)
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
hipError_t fwd_launch(const wcc_desc &d, const void *x, float *coef, float *norm_part,
                      float *max_part, Plan pl, const SelectPrep &prep, const float *wdw, hipStream_t s) {
  if constexpr (!STORE) {
    if (d.act_dtype == WCC_BF16)
      return fwd_launch_t<D, V, STORE>(d, static_cast<const bf16_t *>(x), coef, norm_part, max_part, pl, prep, wdw, s);
  }
  return fwd_launch_t<D, V, STORE>(d, static_cast<const float *>(x), coef, norm_part, max_part, pl, prep, wdw, s);
}

}  // namespace

// Every forward group costs one partial-norm plane (written once, read once): with >= 16
// channels a group that is at most 1/16 of the transform's own traffic.  Measured on gfx950:
// about a thousand waves, each walking as many channels as possible, stream best; more
// groups only pay when a layer has fewer strips than that.
int forward_groups(const wcc_desc &d, int front) {
  const bool busy = front == kFrontChain || arithmetic_bound(d, front == kFrontDw);
  return groups_for(d, d.C_in, busy ? 4096 : 1024, 4);
}

template <bool STORE>
hipError_t fwd_dispatch(const wcc_desc &d, const void *x, float *coef, float *norm_part,
                        float *max_part, Plan pl, const SelectPrep &prep, const float *wdw,
                        hipStream_t s) {
  const bool v4 = d.W % 4 == 0;
  switch (d.levels) {
    case 1: return v4 ? fwd_launch<1, 4, STORE>(d, x, coef, norm_part, max_part, pl, prep, wdw, s)
                      : fwd_launch<1, 2, STORE>(d, x, coef, norm_part, max_part, pl, prep, wdw, s);
    case 2: return fwd_launch<2, 4, STORE>(d, x, coef, norm_part, max_part, pl, prep, wdw, s);
    case 3: return fwd_launch<3, 4, STORE>(d, x, coef, norm_part, max_part, pl, prep, wdw, s);
    case 4: return fwd_launch<4, 4, STORE>(d, x, coef, norm_part, max_part, pl, prep, wdw, s);
  }
  return hipErrorInvalidValue;
}

// G is fixed by the workspace layout (one partial-norm plane per group).  On small layers,
// where even the groups leave fewer than 1024 waves, the four waves of a workgroup split a
// group's channels (if each still gets >= 2).
Plan fwd_plan(const wcc_desc &d, int G) {
  const int Cg = (d.C_in + G - 1) / G;
  const StripMap m = make_map(d, (d.W % 4 == 0) ? 4 : 2);
  const int64_t waves = (int64_t)m.units * d.B * G;
  return Plan{G, waves < 1024 && Cg >= 8, streams(d)};
}

hipError_t launch_haar_fwd(const wcc_desc &d, const float *x, float *coef, float *norm_part, int G,
                           const SelectPrep &prep, hipStream_t s) {
  return fwd_dispatch<true>(d, x, coef, norm_part, nullptr, fwd_plan(d, G), prep, nullptr, s);
}

hipError_t launch_haar_norm(const wcc_desc &d, const void *x, float *norm_part, float *max_part,
                            int G, const SelectPrep &prep, const float *wdw, hipStream_t s) {
  const Plan pl = fwd_plan(d, G);
  return fwd_dispatch<false>(d, x, nullptr, norm_part, max_part, pl, prep, wdw, s);
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
