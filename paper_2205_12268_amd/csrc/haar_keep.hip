// Second transform pass of the fused layer: the kept coefficients go straight to their
// compressed place (Eq. T of the joint shrinkage), optionally as 8-bit codes.
#include "strip_io.h"

namespace wcc {
namespace {

// grid = (ceil(units/4), G, B), block = 256.  DWM as in haar_fwd_kernel.  Q8: xc is int8 codes
// for the clipping parameter q_alpha (> 0) or, if alpha_src is given, for the largest of its
// n_alpha entries (what the selection found as max |kept coefficient|); alpha_slots must be
// null then.
template <int D, int V, int PF, int DWM, bool Q8, class XT, bool NT = false>
__global__ __launch_bounds__(256) void haar_keep_kernel(const XT *__restrict__ x,
                                                        const int32_t *__restrict__ jmap,
                                                        void *__restrict__ xc, float *alpha_slots,
                                                        Geo g, StripMap m, int C, int Cg, int cstep,
                                                        int64_t k, const float *__restrict__ wdw,
                                                        float q_alpha,
                                                        const float *__restrict__ alpha_src,
                                                        int n_alpha, float *alpha_pub) {
  __shared__ float wmax[4];
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int grp = blockIdx.y, b = blockIdx.z;
  LanePos<D> p;
  int row0, col0;
  const bool active = locate<D, V>(m, g, unit, p, row0, col0);
  // the channels of a group: Cg consecutive ones (cstep = 1), or every cstep-th one from grp
  // (cstep = the number of groups)
  const int c0 = cstep == 1 ? grp * Cg : grp;
  const int n_ch = c0 >= C ? 0 : (cstep == 1 ? min(C, c0 + Cg) - c0 : (C - c0 + cstep - 1) / cstep);
  const int64_t kstep = (int64_t)cstep * k;

  using Sink = KeepSink<D, V, Q8>;
  Sink sink(0.f);
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
  if constexpr (Q8) {
    // The clipping parameter the selection found: the largest of its workgroups' maxima.  Taken
    // here, behind the rank loads, so that the two round trips to memory overlap.  The first
    // workgroup leaves it as one float for the contraction that follows.
    if (alpha_src != nullptr) {  // (uniform over the grid)
      q_alpha = alpha_max(alpha_src, n_alpha);
      if (alpha_pub != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
        alpha_pub[0] = q_alpha;
    }
    sink.quant = Quant(q_alpha);
  }
  using Out = typename Sink::Out;
  // (lanes outside the plane read the plane's first rows: a valid address whatever the wave
  // does with them; nothing of theirs is ever stored)
  const XT *src = x + ((size_t)b * C + c0) * g.N + (active ? (size_t)row0 * g.W + col0 : (size_t)0);
  Out *plane = static_cast<Out *>(xc) + ((size_t)b * C + c0) * k;
  // walks the group's channels with whichever sink; returns its max |kept coefficient|
  auto walk = [&](auto &sk, auto &&next_channel) {
    sk.vmax = 0.f;
    sk.aim(plane, k);
    if constexpr (DWM == 0) {
      channel_loop<D, V, PF, NT>(src, g.N * cstep, g.W, n_ch, p, sk, next_channel);
    } else {
      const DwLane q = dw_lane<D, V>(g, m, p, row0, col0);
      channel_loop_dw<D, V, DWM == 2, true, false>(src, wdw + (size_t)c0 * 9, g.N, n_ch, q, p, sk,
                                                   next_channel);
    }
    return sk.vmax;
  };

  float mx = 0.f;
  bool done = false;
  // Dense stores pay where a strip keeps at most half of its slots' worth of positions.  With
  // K_dw folded in and fp32 maps the pass is bound by HBM bytes and the staging measured 5-10 %
  // slower than one store per slot; with bf16 maps it is bound by its arithmetic, and taking
  // the maximum and the store offsets over the list rows instead of over every slot makes it
  // 20 % faster (block at keep 1/8: 375 -> 297 us).
  constexpr int NS = slot_count(D, V);
  constexpr bool kStaged = V == 4 && (D == 2 || D == 3) && (DWM == 0 || sizeof(XT) == 2);
  if constexpr (kStaged) {
    __shared__ uint32_t tiles[4][NS * kWave];
    constexpr int kRankBits = 20;  // list entry = rank | tile index << 20
    int count = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) count += __popcll(__ballot((int)sink.at[s] >= 0));
    const int ni = (count + kWave - 1) / kWave;
    // a wave with lanes outside the plane may stage too (their slots are in no list), except
    // with K_dw folded in, whose border handling counts on the lanes' own columns
    const bool whole = DWM == 0 ? __ballot(active) != 0 : __ballot(active) == ~(uint64_t)0;
    if (whole && n_ch > 0 && ni <= NS / 2 && ni <= 16 && k <= ((int64_t)1 << kRankBits)) {
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
        mx = walk(st, [&plane, k, kstep](auto &sk) {
          sk.flush();
          plane += kstep;
          sk.aim(plane, k);
        });
      };
      if (ni <= 4) run(std::integral_constant<int, 4>{});
      else if (ni <= 8) run(std::integral_constant<int, 8>{});
      else run(std::integral_constant<int, 16>{});  // (ni <= 16 is part of the condition above)
      done = true;
    }
  }
  if (!done && active && n_ch > 0) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
      sink.at[s] = (int)sink.at[s] >= 0 ? sink.at[s] * (uint32_t)sizeof(Out) : Sink::kDropped;
    auto next = [&plane, k, kstep](auto &sk) {
      plane += kstep;
      sk.aim(plane, k);
    };
    if constexpr (Q8) {
      // the quantiser's division path is the same for every value of the layer: one look here
      // instead of one a row inside the channel walk
      if (sink.quant.fast) {
        KeepSink<D, V, Q8, 1> fast(sink);
        mx = walk(fast, next);
      } else {
        KeepSink<D, V, Q8, 2> exact(sink);
        mx = walk(exact, next);
      }
    } else {
      mx = walk(sink, next);
    }
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

template <int D, int V, class XT>
hipError_t keep_launch_t(const wcc_desc &d, int64_t k, const XT *x, const int32_t *jmap, void *xc,
                         float *alpha_slots, Plan pl, const float *wdw, float q_alpha,
                         const float *alpha_src, int n_alpha, float *alpha_pub, hipStream_t s) {
  const Geo g{d.H, d.W, d.levels, (int64_t)d.H * d.W};
  const StripMap m = make_map(d, V);
  const int Cg = (d.C_in + pl.G - 1) / pl.G;
  // Without K_dw in front, group g takes the channels g, g + G, ...: groups running side by
  // side then read neighbouring planes of x and write neighbouring planes of xc (keep pass of
  // workloads 2 and 4 and the stack 2 % faster).  The folded walk indexes its 3x3 weights by
  // consecutive channels and keeps the blocks.
  const int cstep = wdw == nullptr ? pl.G : 1;
  dim3 grid((m.units + 3) / 4, pl.G, d.B);
  const bool q8 = q_alpha > 0.f || alpha_src != nullptr;
#define WCC_KEEP(PF, DWM)                                                                          \
  do {                                                                                             \
    if (q8)                                                                                        \
      hipLaunchKernelGGL((haar_keep_kernel<D, V, PF, DWM, true, XT>), grid, dim3(256), 0, s, x,   \
                         jmap, xc, nullptr, g, m, d.C_in, Cg, cstep, k, wdw, q_alpha, alpha_src, n_alpha, alpha_pub);                    \
    else                                                                                           \
      hipLaunchKernelGGL((haar_keep_kernel<D, V, PF, DWM, false, XT>), grid, dim3(256), 0, s, x,  \
                         jmap, xc, alpha_slots, g, m, d.C_in, Cg, cstep, k, wdw, 0.f, nullptr, 0, nullptr);                    \
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
                         jmap, xc, nullptr, g, m, d.C_in, Cg, cstep, k, wdw, q_alpha, alpha_src, n_alpha, alpha_pub);
    else
      hipLaunchKernelGGL((haar_keep_kernel<D, V, 1, 0, false, XT, true>), grid, dim3(256), 0, s, x,
                         jmap, xc, alpha_slots, g, m, d.C_in, Cg, cstep, k, wdw, 0.f, nullptr, 0, nullptr);
    return hipGetLastError();
  }
  WCC_KEEP(1, 0);
#undef WCC_KEEP
  return hipGetLastError();
}

template <int D, int V>
hipError_t keep_launch(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap, void *xc,
                       float *alpha_slots, Plan pl, const float *wdw, float q_alpha,
                       const float *alpha_src, int n_alpha, float *alpha_pub, hipStream_t s) {
  if (d.act_dtype == WCC_BF16)
    return keep_launch_t<D, V>(d, k, static_cast<const bf16_t *>(x), jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
  return keep_launch_t<D, V>(d, k, static_cast<const float *>(x), jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
}

}  // namespace

hipError_t keep_dispatch(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap, void *xc,
                         float *alpha_slots, Plan pl, const float *wdw, float q_alpha,
                         const float *alpha_src, int n_alpha, float *alpha_pub, hipStream_t s) {
  const bool v4 = d.W % 4 == 0;
  switch (d.levels) {
    case 1: return v4 ? keep_launch<1, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s)
                      : keep_launch<1, 2>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
    case 2: return keep_launch<2, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
    case 3: return keep_launch<3, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
    case 4: return keep_launch<4, 4>(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_haar_keep(const wcc_desc &d, int64_t k, const void *x, const int32_t *jmap,
                            void *xc, float *alpha_slots, const float *wdw, float q_alpha,
                            const float *alpha_src, int n_alpha, float *alpha_pub, hipStream_t s) {
  const Plan pl{groups_for(d, d.C_in, arithmetic_bound(d, wdw != nullptr) ? 4096 : 1024, 4), false,
                streams(d)};
  return keep_dispatch(d, k, x, jmap, xc, alpha_slots, pl, wdw, q_alpha, alpha_src, n_alpha, alpha_pub, s);
}

}  // namespace wcc
