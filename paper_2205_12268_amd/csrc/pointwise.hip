// The 1x1 convolution on the compressed signal (Eq. WCC: K_1x1 applied between T and T^T;
// output channel i is sum_j k_ij x_j over the length-k compressed channel vectors x_j): per sample a
// [C_out x C_in] . [C_in x k] contraction, k contiguous in memory on both sides.
//
// Matrix-core kernel (int8 activation codes):
//   bf16 weights: v_mfma_f32_32x32x16_bf16.  The codes (|n| <= 127) are exact in bf16 and
//                 every product is exact in fp32; only the fp32 accumulation rounds.
//   int8 weights: v_mfma_i32_32x32x32_i8, exact int32 accumulation.
// At the layer's shapes the contraction is bound by HBM (a few tens of flop per byte), so the
// kernel is built around the activation stream: a workgroup owns BM = 128 or 256 output rows
// (all of C_out when it fits, so every activation is read and quantised once) and BN = 128
// positions; each thread loads its share of a 64-channel chunk of the [C_in x BN] activation
// tile (several chunks going out together was measured at every shape and never paid: it costs
// registers, and with them the second workgroup on the compute unit),
// quantises it in registers, transposes 4(n) x CPT(c) patches into LDS, and the waves (wave w
// owns rows 32w..32w+31 and all BN columns) run the MFMAs 64 channels at a time.  As soon as
// a chunk's registers are in LDS the next chunk's loads (activations and weights) are issued,
// so they travel while the MFMAs of this chunk run.  The n rows are stored permuted
// (row (n%NB)*32 + n/NB, NB = BN/32) so that MFMA column c of column block i is n = NB*c + i:
// after the NB column blocks a lane holds NB adjacent n of one output row and stores them as
// one 16- or 8-byte word.  Layers whose kept signal is short would leave most of the chip
// idle with such tiles and turn the kernel into a chain of memory latencies; they take
// smaller tiles (down to 64 x 64), re-reading the activations once per row tile from L2.
// Everything else (fp32 weights, unquantised activations, odd shapes) takes a plain fp32 FMA
// tile kernel on the weights widened to fp32.
#include <type_traits>

#include "wcc_internal.h"

namespace wcc {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int intx4;
typedef __attribute__((__vector_size__(16 * sizeof(int)))) int intx16;

constexpr int BK = 64;

// The layer's alpha: the largest of n partial maxima (n = 1: alpha itself).  The first workgroup
// also publishes it to alpha_out (nullable).  Called by every thread of the workgroup.
__device__ __forceinline__ float load_alpha(const float *__restrict__ alpha, int n, float *alpha_out) {
  const float a = alpha_max(alpha, n);
  if (alpha_out && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
    alpha_out[0] = a;
  return a;
}

// A thread's raw CPT (channels) x 4 (positions) patch of one 64-channel chunk.
// F32: unquantised kept coefficients (16 bytes a channel); else int8 codes (4 bytes a channel).
template <bool F32, int CPT>
struct Patch {
  float4 f[F32 ? CPT : 1];
  uint32_t c[F32 ? 1 : CPT];
  // Loaded through a buffer descriptor of the sample's compressed signal: off is the byte
  // offset of this thread's four positions in the patch's first channel.  No branch, no lane
  // mask: a load never faults (outside the buffer it returns zeros, a wrapped offset lands
  // inside it); what it returns for channels >= C_in meets zero weights (any finite value will
  // do: fp32 coefficients are clipped by the quantiser, and a NaN quantises to a finite level),
  // and for positions >= k it feeds columns that are never stored.
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t xdesc, uint32_t off, int64_t k) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int r = 0; r < CPT; ++r) {
      if constexpr (F32) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(xdesc, off + (uint32_t)r * (uint32_t)k * 4u, 0, 0);
        f[r] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
      } else {
        c[r] = __builtin_amdgcn_raw_buffer_load_b32(xdesc, off + (uint32_t)r * (uint32_t)k, 0, 0);
      }
    }
  }
  // level of channel r, position i, as a float holding an integer in [-127, 127]
  template <bool FAST>
  __device__ __forceinline__ float level(int r, int i, const Quant &q) const {
    if constexpr (F32) {
      const float v = i == 0 ? f[r].x : i == 1 ? f[r].y : i == 2 ? f[r].z : f[r].w;
      return q.template level_as<FAST>(v);
    } else {
      return (float)((int)(c[r] << (24 - 8 * i)) >> 24);
    }
  }
};

// grid = (ceil(k/BN), ceil(M/BM), B), block = 2*BM threads.  Needs k % 4 == 0 and
// K % 8 == 0 (bf16 weights) or K % 16 == 0 (int8 weights).
template <int BM, int BN, bool F32, bool I8W>
__global__ __launch_bounds__(2 * BM) void pointwise_mfma_kernel(
    const void *__restrict__ w, const float *__restrict__ w_scale, const void *__restrict__ xq,
    const float *__restrict__ alpha, int n_alpha, float *alpha_out, float *__restrict__ yc, int M,
    int K, int64_t k, bool stream_out) {
  constexpr int T = 2 * BM;
  constexpr int NB = BN / 32;                // 32-column blocks of the tile: 4 or 2
  constexpr int NG = BN / 4;                 // groups of four positions
  constexpr int CPT = BK / (T / NG);         // channels of a chunk per thread: 4, 8 or 16
  constexpr int ESZ = I8W ? 1 : 2;           // bytes of an LDS element
  constexpr int LDR = I8W ? BK + 16 : (BK + 8) * 2;  // LDS row bytes: 80 / 144 (16-byte aligned,
                                                      // fragment reads free of bank conflicts)
  constexpr int APT = BK * ESZ / 2 / 16;     // 16-byte weight loads per thread and chunk: 2 / 4
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * LDR];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * LDR];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const int b = blockIdx.z;
  const int64_t n0 = (int64_t)blockIdx.x * BN;
  const void *xb = static_cast<const char *>(xq) + (size_t)b * K * k * (F32 ? 4 : 1);
  const unsigned char *wb = static_cast<const unsigned char *>(w);
  const int a_row = t >> 1, a_half = t & 1;  // weight loader: row, which half of the chunk
  const int g = t % NG, kq = t / NG;         // activation loader: n group (4 n), channel group
  const int nchunks = (K + BK - 1) / BK;

  const float al = load_alpha(alpha, n_alpha, alpha_out);
  const Quant quant(al);
  // Both operands are loaded through buffer descriptors (the host has checked that their byte
  // offsets fit 32 bits): weights of rows >= M lie beyond the end and come back
  // as zeros, those of channels >= C_in are sent there by a wave-uniform choice.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  constexpr uint32_t kOutside = 0xFFFFFFF0u;
  const __amdgpu_buffer_rsrc_t wdesc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<unsigned char *>(wb), 0, (int)(uint32_t)((int64_t)M * K * ESZ), 0x00020000);
  const __amdgpu_buffer_rsrc_t xdesc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void *>(xb), 0, (int)(uint32_t)((int64_t)K * k * (F32 ? 4 : 1)), 0x00020000);
  // A workgroup takes the row tiles blockIdx.y, blockIdx.y + gridDim.y, ...: with one workgroup
  // per column tile (gridDim.y = 1) the stores of a row tile drain while the next one is being
  // computed, instead of holding the compute unit until they are out.
  for (int m0 = blockIdx.y * BM; m0 < M; m0 += gridDim.y * BM) {
  // accumulators of the NB column blocks: int32 for int8 weights, fp32 for bf16 weights
  using Acc = std::conditional_t<I8W, intx16, floatx16>;
  Acc acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0;

  // weights of chunk kc: wreg <- w[m0 + a_row][kc*64 + this thread's share], zero outside.
  // They are fetched one chunk ahead (while the MFMAs of the previous chunk run).
  uint4 wreg[APT];
  auto load_w = [&](int kc) {
#pragma unroll
    for (int q = 0; q < APT; ++q) {
      const int kk = kc * BK + (a_half * (BK / 2)) + q * (16 / ESZ);  // first element of the load
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(
          wdesc, kk < K ? (uint32_t)(m0 + a_row) * (uint32_t)(K * ESZ) + (uint32_t)kk * ESZ : kOutside, 0, 0);
      wreg[q] = make_uint4(v.x, v.y, v.z, v.w);
    }
  };

  Patch<F32, CPT> raw;  // the one chunk of activations in flight
  // activations: quantise, transpose the CPT x 4 patch, store with the n rows permuted
  auto stage_patch = [&](const Patch<F32, CPT> &pt, const Quant &quant, auto fast_c) {
    constexpr bool FAST = decltype(fast_c)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t pk[I8W ? (CPT / 4) : (CPT / 2)];
      if constexpr (I8W) {
#pragma unroll
        for (int r = 0; r < CPT; r += 4) {
          const uint32_t c0 = (uint32_t)(int)pt.template level<FAST>(r, i, quant) & 0xFFu;
          const uint32_t c1 = (uint32_t)(int)pt.template level<FAST>(r + 1, i, quant) & 0xFFu;
          const uint32_t c2 = (uint32_t)(int)pt.template level<FAST>(r + 2, i, quant) & 0xFFu;
          const uint32_t c3 = (uint32_t)(int)pt.template level<FAST>(r + 3, i, quant) & 0xFFu;
          pk[r / 4] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
        }
      } else {
#pragma unroll
        for (int r = 0; r < CPT; r += 2) {
          // an integer |v| <= 127 is exact in bf16: its bf16 pattern is the float's high half
          const uint32_t lo = __float_as_uint(pt.template level<FAST>(r, i, quant));
          const uint32_t hi = __float_as_uint(pt.template level<FAST>(r + 1, i, quant));
          pk[r / 2] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
        }
      }
      const int nl = 4 * g + i;  // position inside the tile
      unsigned char *dst = &Bs[((nl % NB) * 32 + nl / NB) * LDR + kq * CPT * ESZ];
      constexpr int words = I8W ? CPT / 4 : CPT / 2;
      if constexpr (words == 8) {
        *reinterpret_cast<uint4 *>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        *reinterpret_cast<uint4 *>(dst + 16) = make_uint4(pk[4], pk[5], pk[6], pk[7]);
      } else if constexpr (words == 4) *reinterpret_cast<uint4 *>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
      else if constexpr (words == 2) *reinterpret_cast<uint2 *>(dst) = make_uint2(pk[0], pk[1]);
      else *reinterpret_cast<uint32_t *>(dst) = pk[0];
    }
  };

  // this thread's four positions in channel kq * CPT of chunk 0
  constexpr uint32_t XB = F32 ? 4u : 1u;  // bytes of an activation
  const uint32_t xoff = ((uint32_t)(kq * CPT) * (uint32_t)k + (uint32_t)(n0 + 4 * g)) * XB;
  load_w(0);
  raw.load(xdesc, xoff, k);
  for (int kc = 0; kc < nchunks; ++kc) {
    {
      if (quant.fast) stage_patch(raw, quant, std::true_type{});
      else stage_patch(raw, quant, std::false_type{});
#pragma unroll
      for (int q = 0; q < APT; ++q)
        *reinterpret_cast<uint4 *>(&As[a_row * LDR + a_half * (BK / 2) * ESZ + q * 16]) = wreg[q];
      __syncthreads();
      // both register tiles are in LDS now: the next chunk travels while this one is multiplied
      // (past the last chunk: zeros and values nobody uses, no memory traffic to speak of)
      load_w(kc + 1);
      raw.load(xdesc, xoff + (uint32_t)((kc + 1) * BK) * (uint32_t)k * XB, k);
      const int fr = lane & 31, half = lane >> 5;
      if constexpr (I8W) {
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
          const intx4 a = __builtin_bit_cast(
              intx4, *reinterpret_cast<const uint4 *>(&As[(wv * 32 + fr) * LDR + ks * 32 + half * 16]));
#pragma unroll
          for (int i = 0; i < NB; ++i) {
            const intx4 bb = __builtin_bit_cast(
                intx4, *reinterpret_cast<const uint4 *>(&Bs[(i * 32 + fr) * LDR + ks * 32 + half * 16]));
            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bb, acc[i], 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
          const bf16x8 a = __builtin_bit_cast(
              bf16x8, *reinterpret_cast<const uint4 *>(&As[(wv * 32 + fr) * LDR + (ks * 16 + half * 8) * 2]));
#pragma unroll
          for (int i = 0; i < NB; ++i) {
            const bf16x8 bb = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4 *>(&Bs[(i * 32 + fr) * LDR + (ks * 16 + half * 8) * 2]));
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc[i], 0, 0, 0);
          }
        }
      }
      __syncthreads();
    }
  }
  // epilogue: acc[i][r] is row (r/4)*8 + (lane/32)*4 + r%4, column NB*(lane%32) + i
  const float sx = al / 127.f;
  const int64_t n = n0 + NB * (lane & 31);
  if (n < k) {  // k % 4 == 0: a lane's NB positions are all inside or all outside
    // The two choices that are the same for the whole wave are taken once, outside the loop over
    // the rows: whether all 32 rows of the wave exist (then no store sits under a test) and
    // whether the output is streamed past the caches.
    auto store_rows = [&](auto whole_c, auto stream_c) {
      constexpr bool WHOLE = decltype(whole_c)::value, STREAM = decltype(stream_c)::value;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wv * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (WHOLE || m < M) {
          float v[NB];
          const float sc = I8W ? sx * w_scale[m] : sx;
#pragma unroll
          for (int i = 0; i < NB; ++i) v[i] = (float)acc[i][r] * sc;
          float *dst = yc + ((size_t)b * M + m) * k + n;
          if constexpr (STREAM) {  // an output that no cache will hold for its reader
            if constexpr (NB == 4) {
              floatx4 o = {v[0], v[1], v[2], v[3]};
              __builtin_nontemporal_store(o, reinterpret_cast<floatx4 *>(dst));
            } else {
              floatx2 o = {v[0], v[1]};
              __builtin_nontemporal_store(o, reinterpret_cast<floatx2 *>(dst));
            }
          } else {
            if constexpr (NB == 4) *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            else *reinterpret_cast<float2 *>(dst) = make_float2(v[0], v[1]);
          }
        }
      }
    };
    const bool whole = m0 + wv * 32 + 32 <= M;
    if (whole) {
      if (stream_out) store_rows(std::true_type{}, std::true_type{});
      else store_rows(std::true_type{}, std::false_type{});
    } else {
      if (stream_out) store_rows(std::false_type{}, std::true_type{});
      else store_rows(std::false_type{}, std::false_type{});
    }
  }  // positions inside the signal
  }  // row tiles
}

template <int BM, int BN, bool I8W>
hipError_t mfma_launch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                       const void *xc, bool f32, const float *alpha, int n_alpha, float *alpha_out,
                       float *yc, hipStream_t s) {
  dim3 grid((unsigned)((k + BN - 1) / BN), (d.C_out + BM - 1) / BM, d.B), block(2 * BM);
  // several row tiles: one workgroup walks them all where the column tiles alone fill the chip
  if (grid.y > 1 && (int64_t)grid.x * grid.z >= 2 * 256) grid.y = 1;
  // The inverse transform reads yc next.  Up to about twice the 256 MB memory-side cache it is
  // better left there (measured); beyond that the output is streamed past it.
  const bool stream_out = (int64_t)d.B * d.C_out * k * 4 > ((int64_t)512 << 20);
  if (f32)
    hipLaunchKernelGGL((pointwise_mfma_kernel<BM, BN, true, I8W>), grid, block, 0, s, w, w_scale,
                       xc, alpha, n_alpha, alpha_out, yc, d.C_out, d.C_in, k, stream_out);
  else
    hipLaunchKernelGGL((pointwise_mfma_kernel<BM, BN, false, I8W>), grid, block, 0, s, w, w_scale,
                       xc, alpha, n_alpha, alpha_out, yc, d.C_out, d.C_in, k, stream_out);
  return hipGetLastError();
}

// ---- the contraction where it is bound by arithmetic (hundreds of channels and more) ------------
// The kernel above is laid out for the memory-bound layers: a wave tile of 32 x 128 re-reads
// every activation fragment in all eight waves (five 16-byte LDS reads per four matrix
// instructions) and one LDS buffer costs two barriers a chunk.  With C_in in the hundreds or
// thousands the matrix cores are what counts, so this variant spends LDS bandwidth and barriers
// sparingly:
//   workgroup tile 128 (rows) x 128 (positions), four waves in a 2 x 2 arrangement, wave tile
//   64 x 64 = 2 x 2 blocks of 32 x 32 (64 accumulator registers, so that two register sets of
//   loads in flight still leave room for three workgroups a compute unit): four fragment reads
//   per four matrix instructions;
//   two LDS stages of 64 bytes of K a row (32 channels of bf16, 64 of int8: the byte addressing
//   of both operand types is the same), 20 KB each: while the matrix instructions of stage s
//   run, the registers loaded two stages earlier are converted and written into the other
//   buffer and the loads of the stage after next are issued; one barrier a stage.
// Activations are int8 codes only (the fused layer's default route).  Positions are stored
// permuted inside a wave's 64 columns (row (n % 2) * 32 + n / 2), so that after the two column
// blocks a lane holds two adjacent positions of one output row and stores 8 bytes.
// Which tile a workgroup takes: the hardware hands consecutive workgroups to the 8 dies in
// turn, each die with an L2 of its own; here die x works through the x-th eighth of the tile
// list (positions fastest, then rows, then samples), so that the tiles a die has in flight share
// their activation columns and walk through neighbouring weight rows in ITS L2.  With the
// natural order every die touches every operand and most fetches come from beyond the L2s
// (1.1 GB at 5 TB/s for 116 GFLOP on 4096 x 1024 weights).
// Needs k % 4 == 0 and C_in % 8 == 0 (bf16 weights) or % 16 == 0 (int8 weights).
constexpr int kDies = 8;
constexpr int kTileM = 128, kTileN = 128, kTileKB = 64, kTileLDR = kTileKB + 16;
constexpr int kTileMinChannels = 256;

// WM: 32-row blocks of a wave tile, 2 (workgroup tile 128 rows) or 4 (256 rows)
template <bool I8W, int WM>
__global__ __launch_bounds__(256, WM == 2 ? 3 : 2) void pointwise_tile_kernel(
    const void *__restrict__ w, const float *__restrict__ w_scale, const int8_t *__restrict__ xq,
    const float *__restrict__ alpha, int n_alpha, float *alpha_out, float *__restrict__ yc, int M,
    int K, int64_t k, bool stream_out, int gx, int gy, int tiles, int dies) {
  constexpr int ESZ = I8W ? 1 : 2;        // bytes of a weight / of an activation in LDS
  constexpr int KC = kTileKB / ESZ;       // channels a stage: 64 or 32
  constexpr int CPT = KC / 8;             // channels a thread converts: 8 or 4
  constexpr int LDR = kTileLDR;
  constexpr int TM = 64 * WM;             // rows of the workgroup tile
  constexpr int WQ = WM / 2;              // 16-byte weight loads a thread and stage: half a row, or a whole one
  __shared__ __attribute__((aligned(16))) unsigned char As[2][TM * LDR];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[2][kTileN * LDR];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const int wm = wv >> 1, wn = wv & 1;    // the wave's place in the 2 x 2 arrangement
  // grid = 8 * ceil(tiles / 8) workgroups in one dimension
  // (dies = 1: the natural order, for layers whose weights every L2 holds anyway and whose time
  // goes into writing yc: there the dies had better write one neighbourhood together)
  const int tile = (blockIdx.x % dies) * (gridDim.x / dies) + blockIdx.x / dies;
  const int b = tile / (gx * gy), by = (tile / gx) % gy, bx = tile % gx;
  const int64_t n0 = (int64_t)bx * kTileN;
  const int m0 = by * TM;
  const int8_t *xb = xq + (size_t)b * K * k;
  const unsigned char *wb = static_cast<const unsigned char *>(w);
  // activation loader: group of four positions, channel group.  A wave takes 8 position groups
  // x all 8 channel groups: the 32 lanes that an LDS write serves together then hit 8 rows
  // (160 bytes apart) x 4 channel groups (8 bytes apart) = 32 different 8-byte bank pairs; with
  // 32 position groups a wave the same write was a four-way bank conflict.
  const int g = wv * 8 + (lane & 7), kq = lane >> 3;
  const int stages = (K + KC - 1) / KC;

  const float al = alpha_max(alpha, n_alpha);  // (every thread of the workgroup is here)
  if (alpha_out && tile == 0 && threadIdx.x == 0) alpha_out[0] = al;
  if (tile >= tiles) return;  // the workgroups that pad the grid to a multiple of 8

  using Acc = std::conditional_t<I8W, intx16, floatx16>;
  Acc acc[WM][2];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  // global -> registers: half a weight row (32 of a stage's 64 bytes of K; two threads a row)
  // and the thread's CPT x 4 activation patch,
  // through buffer descriptors of the weights and of the sample's compressed signal: what lies
  // a load never faults (outside the buffer it returns zeros, and an offset that wraps lands
  // inside it), so there is no branch and no lane mask, a prefetch may run past the last
  // stage, and the compiler can count the loads in flight exactly.  Weights of channels
  // >= C_in are zeros (the offset is sent outside, a wave-uniform choice), so whatever the
  // activation loads return for those channels is multiplied by zero; rows >= M and positions
  // >= k (last tiles) read something, but their rows and columns are never stored and feed
  // no other.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  struct Regs {
    u32x4 w[2 * WQ];
    uint32_t x[CPT];
  };
  const __amdgpu_buffer_rsrc_t wdesc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<unsigned char *>(wb), 0, (int)(uint32_t)((int64_t)M * K * ESZ), 0x00020000);
  const __amdgpu_buffer_rsrc_t xdesc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int8_t *>(xb), 0, (int)(uint32_t)((int64_t)K * k), 0x00020000);
  constexpr uint32_t kOutside = 0xFFFFFFF0u;
  // (two lanes a row: their 16-byte LDS writes collide pairwise with those of other rows, but a
  // row per lane -- conflict-free in LDS -- makes every load touch 64 cache lines instead of 32
  // and was measured slower, 175 vs 147 us)
  const int a_row = WM == 2 ? t >> 1 : t, a_half = WM == 2 ? t & 1 : 0;
  const uint32_t wrow = (uint32_t)(m0 + a_row) * (uint32_t)(K * ESZ);
  const uint32_t xcol = (uint32_t)(n0 + 4 * g) + (uint32_t)(kq * CPT) * (uint32_t)k;
  auto fetch = [&](Regs &r, int st) {
#pragma unroll
    for (int q = 0; q < 2 * WQ; ++q) {
      // first channel of the 16-byte load; a stage is whole or empty in K (C_in is a multiple of
      // what 16 bytes hold), but its two halves may differ: the choice is the lane's
      const int kk = st * KC + (a_half * 2 + q) * (16 / ESZ);
      r.w[q] = __builtin_amdgcn_raw_buffer_load_b128(wdesc, kk < K ? wrow + (uint32_t)kk * ESZ : kOutside, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c)  // channel st * KC + c (+ kq * CPT, which xcol carries)
      r.x[c] = __builtin_amdgcn_raw_buffer_load_b32(xdesc, xcol + (uint32_t)(st * KC + c) * (uint32_t)k, 0, 0);
  };
  // registers -> LDS stage `buf`: the weight row as it is; the patch transposed (and widened to
  // bf16 for bf16 weights: an integer |v| <= 127 is exact there, its pattern is the float's
  // high half), 8 bytes of K for each of the four positions
  auto stash = [&](const Regs &r, int buf) {
#pragma unroll
    for (int q = 0; q < 2 * WQ; ++q)
      *reinterpret_cast<u32x4 *>(&As[buf][a_row * LDR + (a_half * 2 + q) * 16]) = r.w[q];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t lo, hi;
      if constexpr (I8W) {
        // byte i of eight channel words -> two words of four channels each
        const uint32_t sel = 0x0C0C0400u + 0x00000101u * i;   // {.., .., b[i], a[i]}
        const uint32_t p01 = __builtin_amdgcn_perm(r.x[1], r.x[0], sel);
        const uint32_t p23 = __builtin_amdgcn_perm(r.x[3], r.x[2], sel);
        const uint32_t p45 = __builtin_amdgcn_perm(r.x[5], r.x[4], sel);
        const uint32_t p67 = __builtin_amdgcn_perm(r.x[7], r.x[6], sel);
        lo = (p01 & 0xFFFFu) | (p23 << 16);
        hi = (p45 & 0xFFFFu) | (p67 << 16);
      } else {
        float f[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) f[c] = (float)((int)(r.x[c] << (24 - 8 * i)) >> 24);
        lo = __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);
        hi = __builtin_amdgcn_perm(__float_as_uint(f[3]), __float_as_uint(f[2]), 0x07060302u);
      }
      const int nl = 4 * g + i;  // position inside the workgroup's tile
      const int row = (nl & 64) + (nl & 1) * 32 + ((nl & 63) >> 1);
      *reinterpret_cast<uint2 *>(&Bs[buf][row * LDR + kq * 8]) = make_uint2(lo, hi);
    }
  };
  const int fr = lane & 31, half = lane >> 5;
  auto multiply = [&](int buf) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      uint4 a[WM], bb[2];
#pragma unroll
      for (int i = 0; i < WM; ++i)
        a[i] = *reinterpret_cast<const uint4 *>(&As[buf][(wm * (32 * WM) + i * 32 + fr) * LDR + ks * 32 + half * 16]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        bb[j] = *reinterpret_cast<const uint4 *>(&Bs[buf][(wn * 64 + j * 32 + fr) * LDR + ks * 32 + half * 16]);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          if constexpr (I8W)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(intx4, a[i]),
                                                             __builtin_bit_cast(intx4, bb[j]), acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                               __builtin_bit_cast(bf16x8, bb[j]), acc[i][j], 0, 0, 0);
        }
    }
  };

  // Two register sets: the loads of a stage are issued two stages before they are converted,
  // so that they have a whole stage of matrix instructions (and the other workgroup's) to
  // arrive.  r0 carries the odd stages, r1 the even ones.
  Regs r0, r1;
  fetch(r0, 0);
  stash(r0, 0);
  fetch(r0, 1);
  fetch(r1, 2);
  __syncthreads();
  // (an odd number of stages is rounded up: the stage past the end loads zeros and adds them;
  // a way out in the middle of the loop body made the compiler keep two copies of the
  // accumulators and move 64 registers a stage)
  for (int s = 0; s < stages; s += 2) {
    stash(r0, 1);      // stage s + 1 (every wave left buffer 1 at the last barrier)
    fetch(r0, s + 3);
    multiply(0);       // stage s
    __syncthreads();
    // (nothing of the next half moves up across this point: the compiler would start converting
    // r1 here, a stage early, and wait for loads that have another stage to arrive)
    __builtin_amdgcn_sched_barrier(0);
    stash(r1, 0);      // stage s + 2
    fetch(r1, s + 4);
    multiply(1);       // stage s + 1
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  }

  // acc[i][j][r]: row wm*64 + i*32 + (r/4)*8 + (lane/32)*4 + r%4, position wn*64 + 2*(lane%32) + j
  const float sx = al / 127.f;
  const int64_t n = n0 + wn * 64 + 2 * fr;
  if (n < k) {  // k % 4 == 0 and n even: both positions inside or both outside
    // (what is the same for the whole wave is decided once, outside the loops over the rows)
    auto store_rows = [&](auto whole_c, auto stream_c) {
      constexpr bool WHOLE = decltype(whole_c)::value, STREAM = decltype(stream_c)::value;
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * (32 * WM) + i * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (WHOLE || m < M) {
            const float sc = I8W ? sx * w_scale[m] : sx;
            const float v0 = (float)acc[i][0][r] * sc, v1 = (float)acc[i][1][r] * sc;
            float *dst = yc + ((size_t)b * M + m) * k + n;
            if constexpr (STREAM) {
              floatx2 o = {v0, v1};
              __builtin_nontemporal_store(o, reinterpret_cast<floatx2 *>(dst));
            } else {
              *reinterpret_cast<float2 *>(dst) = make_float2(v0, v1);
            }
          }
        }
    };
    const bool whole = m0 + wm * (32 * WM) + 32 * WM <= M;
    if (whole) {
      if (stream_out) store_rows(std::true_type{}, std::true_type{});
      else store_rows(std::true_type{}, std::false_type{});
    } else {
      if (stream_out) store_rows(std::false_type{}, std::true_type{});
      else store_rows(std::false_type{}, std::false_type{});
    }
  }
}

template <bool I8W, int WM>
hipError_t tile_launch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale, const void *xc,
                       const float *alpha, int n_alpha, float *alpha_out, float *yc, hipStream_t s) {
  constexpr int TM = 64 * WM;
  const int64_t gx = (k + kTileN - 1) / kTileN, gy = (d.C_out + TM - 1) / TM;
  const int64_t tiles = gx * gy * d.B;
  if (tiles > (int64_t)1 << 30) return hipErrorInvalidValue;
  dim3 grid((unsigned)((tiles + kDies - 1) / kDies * kDies)), block(256);
  const bool stream_out = (int64_t)d.B * d.C_out * k * 4 > ((int64_t)512 << 20);
  hipLaunchKernelGGL((pointwise_tile_kernel<I8W, WM>), grid, block, 0, s, w, w_scale,
                     static_cast<const int8_t *>(xc), alpha, n_alpha, alpha_out, yc, d.C_out, d.C_in, k,
                     stream_out, (int)gx, (int)gy, (int)tiles,
                     (int64_t)d.C_out * d.C_in * (I8W ? 1 : 2) >= ((int64_t)1 << 20) ? kDies : 1);
  return hipGetLastError();
}

// Is the layer one for the arithmetic-bound variant?  int8 codes in, enough channels that the
// matrix instructions outweigh the stream (measured crossover), at least a tile of output
// rows, and a workgroup for every compute unit.
static bool wants_tile_kernel(const wcc_desc &d, int64_t k, bool f32) {
  if (f32 || d.C_in < kTileMinChannels || d.C_out < kTileM) return false;
  // an expansion layer with few input channels spends its time writing yc: the stream kernel's
  // 16-byte stores and its walk over the row tiles do that better (1024 x 256: 170 vs 180 us)
  if (d.C_in < 512 && d.C_out >= 4 * d.C_in) return false;
  const int64_t wgs = ((k + kTileN - 1) / kTileN) * ((d.C_out + kTileM - 1) / kTileM) * (int64_t)d.B;
  // (byte offsets into the weights and into a sample's compressed signal fit 32 bits)
  const int64_t limit = (int64_t)0xFFFFFFF0;
  if ((int64_t)(d.C_out + kTileM) * d.C_in * 2 > limit || (int64_t)d.C_in * k > limit) return false;
  return wgs >= 256 && wgs <= ((int64_t)1 << 30);
}

// Tile choice.  Large tiles first (BM = 256 when C_out needs it: every activation is then read
// once), as long as they give every compute unit a workgroup; otherwise smaller ones.
template <bool I8W>
hipError_t mfma_dispatch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                         const void *xc, bool f32, const float *alpha, int n_alpha, float *alpha_out,
                         float *yc, hipStream_t s) {
#define WCC_MFMA(BM_, BN_) \
  return mfma_launch<BM_, BN_, I8W>(d, k, w, w_scale, xc, f32, alpha, n_alpha, alpha_out, yc, s)
  // (WM = 4, 256-row tiles with 128 x 64 wave tiles, two workgroups a compute unit: measured
  // slower on every layer tried, 176 vs 147 us at 1024 -> 4096 channels; three resident
  // workgroups hide more than the halved conversion work saves)
  if (wants_tile_kernel(d, k, f32))
    return tile_launch<I8W, 2>(d, k, w, w_scale, xc, alpha, n_alpha, alpha_out, yc, s);
  const int64_t want = 256;  // compute units
  auto wgs = [&](int bm, int bn) {
    return ((k + bn - 1) / bn) * ((d.C_out + bm - 1) / bm) * (int64_t)d.B;
  };
  if (d.C_out > 128 && wgs(256, 128) >= want) WCC_MFMA(256, 128);
  if (d.C_out <= 128 && wgs(128, 128) >= want) WCC_MFMA(128, 128);
  // (a quarter of the chip is enough for the 128-row tile: on the short signals of deep layers
  // the smaller tile quantises and stages every activation once more per extra row tile, which
  // costs more than the idle units: 960 -> 320 channels at k = 512, 19.5 -> 17.2 us)
  if (d.C_out > 64 && wgs(128, 64) >= want / 4) WCC_MFMA(128, 64);
  WCC_MFMA(64, 64);
#undef WCC_MFMA
}

// ---- plain fp32 FMA tile kernel (any storage types, any shape) ------------------------------------
template <int DT> struct WLoad;
template <> struct WLoad<WCC_F32> {
  static __device__ __forceinline__ float at(const void *w, size_t i) { return static_cast<const float *>(w)[i]; }
};
template <> struct WLoad<WCC_BF16> {
  static __device__ __forceinline__ float at(const void *w, size_t i) {
    return __uint_as_float((uint32_t) static_cast<const uint16_t *>(w)[i] << 16);
  }
};
template <> struct WLoad<WCC_I8> {
  static __device__ __forceinline__ float at(const void *w, size_t i) { return (float)static_cast<const int8_t *>(w)[i]; }
};

constexpr int FT = 64, FK = 16;

// grid = (ceil(k/64), ceil(M/64), B), block = 256; thread (ty, tx) computes rows ty*4..+3 and
// columns tx, tx+16, tx+32, tx+48 of the tile; channels are accumulated in increasing order.
// XM: 0 = fp32 activations as they are, 1 = int8 codes, 2 = fp32 activations quantised on load
template <int WDT, int XM>
__global__ __launch_bounds__(256) void pointwise_fma_kernel(const void *__restrict__ w,
                                                            const float *__restrict__ w_scale,
                                                            const void *__restrict__ xc,
                                                            const float *__restrict__ alpha,
                                                            int n_alpha, float *alpha_out,
                                                            float *__restrict__ yc, int M, int K,
                                                            int64_t k) {
  __shared__ float Ws[FK][FT + 1];
  __shared__ float Xs[FK][FT];
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int b = blockIdx.z, m0 = blockIdx.y * FT;
  const int64_t n0 = (int64_t)blockIdx.x * FT;
  float acc[4][4] = {};
  const float al = XM != 0 ? load_alpha(alpha, n_alpha, alpha_out) : 0.f;
  const Quant quant(al);
  for (int k0 = 0; k0 < K; k0 += FK) {
    // Ws[kk][mm] = w[m0 + mm][k0 + kk]
    for (int e = t; e < FT * FK; e += 256) {
      const int mm = e / FK, kk = e % FK;
      float v = 0.f;
      if (m0 + mm < M && k0 + kk < K) v = WLoad<WDT>::at(w, (size_t)(m0 + mm) * K + k0 + kk);
      Ws[kk][mm] = v;
    }
    for (int e = t; e < FT * FK; e += 256) {
      const int kk = e / FT, nn = e % FT;
      float v = 0.f;
      if (k0 + kk < K && n0 + nn < k) {
        const size_t at = ((size_t)b * K + k0 + kk) * k + n0 + nn;
        if (XM == 1) v = (float)static_cast<const int8_t *>(xc)[at];
        else if (XM == 2) v = quant.level(static_cast<const float *>(xc)[at]);
        else v = static_cast<const float *>(xc)[at];
      }
      Xs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FK; ++kk) {
      float a[4], x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = Ws[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) x[j] = Xs[kk][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], x[j], acc[i][j]);
    }
    __syncthreads();
  }
  const float sx = XM != 0 ? al / 127.f : 1.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
    const float sc = sx * (WDT == WCC_I8 ? w_scale[m] : 1.f);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t n = n0 + tx + 16 * j;
      if (n < k) yc[((size_t)b * M + m) * k + n] = acc[i][j] * sc;
    }
  }
}

template <int WDT, int XM>
hipError_t fma_launch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                      const void *xc, const float *alpha, int n_alpha, float *alpha_out, float *yc,
                      hipStream_t s) {
  dim3 grid((unsigned)((k + FT - 1) / FT), (d.C_out + FT - 1) / FT, d.B);
  hipLaunchKernelGGL((pointwise_fma_kernel<WDT, XM>), grid, dim3(256), 0, s, w, w_scale, xc, alpha,
                     n_alpha, alpha_out, yc, d.C_out, d.C_in, k);
  return hipGetLastError();
}

template <int WDT>
hipError_t fma_dispatch(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                        const void *xc, int xm, const float *alpha, int n_alpha, float *alpha_out,
                        float *yc, hipStream_t s) {
  switch (xm) {
    case 0: return fma_launch<WDT, 0>(d, k, w, w_scale, xc, alpha, n_alpha, alpha_out, yc, s);
    case 1: return fma_launch<WDT, 1>(d, k, w, w_scale, xc, alpha, n_alpha, alpha_out, yc, s);
    default: return fma_launch<WDT, 2>(d, k, w, w_scale, xc, alpha, n_alpha, alpha_out, yc, s);
  }
}

}  // namespace

hipError_t launch_pointwise(const wcc_desc &d, int64_t k, const void *w, const float *w_scale,
                            const void *xc, bool xc_is_f32, const float *alpha, int n_alpha,
                            float *alpha_out, float *yc, hipStream_t s) {
  const bool quant = d.act_quant_bits == 8;
  const int K = d.C_in;
  // the matrix-core kernels address the activations and the weights with 32-bit byte offsets
  // (4 GB of weights or of one sample's compressed signal take the plain kernel below)
  const int64_t limit = (int64_t)0xFFFFFFF0;
  const bool narrow = (int64_t)(d.C_out + 256) * K * 2 <= limit && (int64_t)K * k * (xc_is_f32 ? 4 : 1) <= limit;
  if (!narrow) {
  } else if (quant && d.w_dtype == WCC_BF16 && K % 8 == 0 && k % 4 == 0)
    return mfma_dispatch<false>(d, k, w, w_scale, xc, xc_is_f32, alpha, n_alpha, alpha_out, yc, s);
  else if (quant && d.w_dtype == WCC_I8 && K % 16 == 0 && k % 4 == 0)
    return mfma_dispatch<true>(d, k, w, w_scale, xc, xc_is_f32, alpha, n_alpha, alpha_out, yc, s);
  const int xm = !quant ? 0 : (xc_is_f32 ? 2 : 1);
  switch (d.w_dtype) {
    case WCC_F32: return fma_dispatch<WCC_F32>(d, k, w, w_scale, xc, xm, alpha, n_alpha, alpha_out, yc, s);
    case WCC_BF16: return fma_dispatch<WCC_BF16>(d, k, w, w_scale, xc, xm, alpha, n_alpha, alpha_out, yc, s);
    case WCC_I8: return fma_dispatch<WCC_I8>(d, k, w, w_scale, xc, xm, alpha, n_alpha, alpha_out, yc, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace wcc
