// C ABI of libwcc: argument checks, workspace carving, and the order in which the kernels of
// Alg. 1 are enqueued.  No arithmetic of the method happens on the host.
#include <mutex>
#include <new>

#include "wcc_internal.h"

// Scratch memory of wcc_forward_static, inside the library's device image: every GPU the library
// runs on holds its own copy at its own address until the process ends.  Host code never uses
// the array's name as an address; static_scratch_of() asks the runtime where the current
// device's copy lives, once per device.
static __device__ __align__(256) unsigned char scratch[WCC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on device i (nullptr: not asked yet)

// Address of `scratch` on `device`, which must be the current device.
hipError_t static_scratch_of(int device, void **out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] == nullptr) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}
}  // namespace

struct wcc_ctx {
  int device = 0;               // the device wcc_create was given: owner of static_ws
  void *static_ws = nullptr;    // that device's copy of `scratch`
  void *ws = nullptr;
  size_t ws_bytes = 0;
  bool profiling = false;
  bool have_times = false;
  hipEvent_t ev[WCC_T_COUNT][2] = {};
  bool ev_ok = false;
  bool marked[WCC_T_COUNT] = {};  // stage bracket recorded since profiling was switched on
  int block_profile_layer = 1;  // which layer of wcc_block_forward the stage events bracket
};

#define WCC_TRY(expr)                                 \
  do {                                                \
    if ((expr) != hipSuccess) return WCC_ERR_HIP;     \
  } while (0)

namespace wcc {
namespace {

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

constexpr int64_t kEarlyAlphaMinPositions = 16384;  // (the one-workgroup selection's limit)
constexpr int64_t kEarlyAlphaMinKept = (int64_t)4 << 20;

wcc_status check_desc(const wcc_desc *d) {
  if (!d) return WCC_ERR_NULL;
  if (d->B < 1 || d->C_in < 1 || d->C_out < 1 || d->H < 2 || d->W < 2) return WCC_ERR_SHAPE;
  if (d->levels < 1 || d->levels > kMaxLevels) return WCC_ERR_SHAPE;
  const int s = 1 << d->levels;
  if (d->H % s || d->W % s) return WCC_ERR_SHAPE;
  // grid limits and 32-bit in-plane offsets
  if (d->B > 65535 || d->C_in > 65535 || d->C_out > 65535) return WCC_ERR_SHAPE;
  // (a plane's bytes, and an offset that lies beyond every plane, fit 32 bits: strip.h, kRowDropped)
  if ((int64_t)d->H * d->W > ((int64_t)1 << 30) - 16) return WCC_ERR_SHAPE;
  if (d->w_dtype != WCC_F32 && d->w_dtype != WCC_BF16 && d->w_dtype != WCC_I8 && d->w_dtype != WCC_I4)
    return WCC_ERR_DTYPE;
  if (d->w_dtype == WCC_I4 && d->C_in % 2) return WCC_ERR_SHAPE;
  if (d->act_quant_bits != 0 && d->act_quant_bits != 8) return WCC_ERR_DTYPE;
  if (d->act_dtype != WCC_F32 && d->act_dtype != WCC_BF16) return WCC_ERR_DTYPE;
  if (d->norm != WCC_NORM_L1 && d->norm != WCC_NORM_L2) return WCC_ERR_DTYPE;
  if (d->norm == WCC_NORM_L2 && d->act_dtype != WCC_F32) return WCC_ERR_UNSUPPORTED;
  if (d->keep_num < 1 || d->keep_den < 1 || d->keep_num > d->keep_den) return WCC_ERR_KEEP;
  const int64_t N = (int64_t)d->H * d->W;
  // keep_num * N must not overflow
  if (d->keep_num > (INT64_MAX - d->keep_den) / N) return WCC_ERR_KEEP;
  const int64_t k = (d->keep_num * N + d->keep_den - 1) / d->keep_den;
  if (k < 1 || k > N) return WCC_ERR_KEEP;
  return WCC_OK;
}

int64_t k_of(const wcc_desc &d) {
  const int64_t N = (int64_t)d.H * d.W;
  return (d.keep_num * N + d.keep_den - 1) / d.keep_den;
}

// integer weight codes with a per-output-channel scale
bool coded(int w_dtype) { return w_dtype == WCC_I8 || w_dtype == WCC_I4; }

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

wcc_status need_ws(const wcc_ctx *ctx, const WsLayout &L) {
  if (!ctx->ws || ctx->ws_bytes < L.total) return WCC_ERR_WORKSPACE;
  return WCC_OK;
}

}  // namespace

// fewest select workgroups a launch should have (two a compute unit: with fewer the passes
// get slower again: measured at 256 and 480 workgroups)
constexpr size_t kSelectMinBlocks = 512;

WsLayout ws_layout(const wcc_desc &d, int front) {
  WsLayout L{};
  const size_t N = (size_t)d.H * d.W, B = d.B, k = (size_t)k_of(d);
  L.G = forward_groups(d, front);
  // select workgroups take 1024, 2048 or 4096 keys: the most that still leaves kSelectMinBlocks
  // of them (fewer, fatter workgroups merge fewer histograms and read the previous pass's
  // histogram less often)
  L.sel_slots = 1;
  for (int sl = 4; sl > 1; sl /= 2)
    if ((N + (size_t)kSelectChunk * sl - 1) / ((size_t)kSelectChunk * sl) * B >= kSelectMinBlocks) { L.sel_slots = sl; break; }
  L.nblk = (int)((N + (size_t)kSelectChunk * L.sel_slots - 1) / ((size_t)kSelectChunk * L.sel_slots));
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  L.norm_part = take((size_t)L.G * B * N * 4);
  L.max_part = take(d.act_quant_bits == 8 ? (size_t)L.G * B * N * 4 : 0);
  L.norm = take(B * N * 4);
  L.hist = take(B * 3 * kRadixBins * 4);
  L.state = take(B * sizeof(SelectState));
  L.block_sfx = take(B * (size_t)L.nblk * kSfxStride * 2);
  L.block_gthi = take(B * (size_t)L.nblk * 4);
  L.jmap = take(B * N * 4);
  L.idx = take(B * k * 4);
  L.alpha = take(256);
  L.block_top = take(d.act_quant_bits == 8 ? B * (size_t)L.nblk * 4 : 0);
  L.scratch = take(kInvScratchBytes);
  L.xc32 = take(B * (size_t)d.C_in * k * 4);
  L.yc = take(B * (size_t)d.C_out * k * 4);
  L.w8 = take(d.w_dtype == WCC_I4 ? (size_t)d.C_out * d.C_in : 0);
  L.total = off;
  return L;
}


// The contraction, with 4-bit weight codes widened to int8 in the workspace first.
hipError_t pointwise_any(char *ws, const WsLayout &L, const wcc_desc &d, int64_t k, const void *w,
                         const float *w_scale, const void *xc, bool xc_is_f32, const float *alpha,
                         int n_alpha, float *alpha_out, float *yc, hipStream_t s) {
  if (d.w_dtype != WCC_I4)
    return launch_pointwise(d, k, w, w_scale, xc, xc_is_f32, alpha, n_alpha, alpha_out, yc, s);
  int8_t *w8 = reinterpret_cast<int8_t *>(ws + L.w8);
  const hipError_t e = launch_unpack_i4(static_cast<const uint8_t *>(w), w8, (int64_t)d.C_out * d.C_in, s);
  if (e != hipSuccess) return e;
  wcc_desc d8 = d;
  d8.w_dtype = WCC_I8;
  return launch_pointwise(d8, k, w8, w_scale, xc, xc_is_f32, alpha, n_alpha, alpha_out, yc, s);
}

// Where the index set I of a layer comes from.
enum { kListSelect = 0,  // joint shrinkage: top-k channel norms (Alg. 1)
       kListPrefix = 1,  // the first k positions of the wavelet vector, whatever the input
       kListGiven = 2 }; // the caller's list

// One WCC layer (Alg. 1 with the quantiser) on a workspace that starts at `ws`.  residual
// (nullable, [B, C_out, H, W]) is added to the output by the last kernel.  wdw (nullable,
// [C_in, 3, 3]): the layer's input is K_dw x, convolved on the fly by both transform passes; with
// src given (x unused) it is K_dw t1, t1 rebuilt from a producer layer's compressed output.
// stop_before_inverse: the layer ends with Y_wt in its workspace (y unused), for a consumer that
// takes it from there.  prof: bracket the stages with the context's events.
wcc_status forward_on(wcc_ctx *ctx, char *ws, const WsLayout &L, const wcc_desc &d, const void *x,
                      const void *w, const float *w_scale, float alpha_in, void *y,
                      int32_t *idx_out, float *alpha_out_dev, const void *residual,
                      const float *wdw, bool prof, hipStream_t s, int list = kListSelect,
                      const int32_t *idx_given = nullptr, const ChainSrc *src = nullptr,
                      bool stop_before_inverse = false) {
  const int64_t k = k_of(d);
  const bool quant = d.act_quant_bits == 8;

  float *part = reinterpret_cast<float *>(ws + L.norm_part);
  float *norm = reinterpret_cast<float *>(ws + L.norm);
  int32_t *jmap = reinterpret_cast<int32_t *>(ws + L.jmap);
  int32_t *idx = idx_out ? idx_out : reinterpret_cast<int32_t *>(ws + L.idx);
  float *slots = reinterpret_cast<float *>(ws + L.alpha);
  float *xc32 = reinterpret_cast<float *>(ws + L.xc32);
  float *yc = reinterpret_cast<float *>(ws + L.yc);

  auto mark = [&](int stage, int which) -> hipError_t {
    if (!prof) return hipSuccess;
    ctx->marked[stage] = true;
    return hipEventRecord(ctx->ev[stage][which], s);
  };

  // Where the clipping parameter comes from decides in which form the kept coefficients travel.
  //   caller's alpha:  the second pass decides the codes itself, int8 leaves the chip;
  //   selected list:   the first pass also keeps max_c |coefficient| per position and the
  //                    selection's last kernel reduces it over the positions each of its
  //                    workgroups keeps (block_top), so alpha is known before the second pass,
  //                    which again decides the codes itself;
  //   fixed list (no first pass), k % 4 != 0 (the contraction reads four codes a word), or more
  //   workgroup maxima than a consumer should have to combine:
  //                    the second pass writes fp32 and raises the slots, the contraction's
  //                    loader quantises.
  const bool given = quant && alpha_in > 0.f;
  const int n_top = select_top_count(d, L);
  // (small layers -- a plane that the one-workgroup selection takes and a few million kept
  // coefficients at most -- stay on the fp32 route: they are bound by launches, not bytes, and
  // the extra loads of the maxima only lengthen them: measured on the 16-layer stack, 869 vs
  // 851 us at keep 1/4)
  const bool small_layer = (int64_t)d.H * d.W <= kEarlyAlphaMinPositions &&
                           (int64_t)d.B * d.C_in * k < kEarlyAlphaMinKept;
  const bool early = quant && !given && list == kListSelect && k % 4 == 0 && n_top <= 8192 && !small_layer;
  const bool codes_now = early || (given && k % 4 == 0);
  float *tops = reinterpret_cast<float *>(ws + L.block_top);
  // the contraction finds alpha in the slots: as the largest of them, or (early) as the one
  // float the second pass left there after combining the selection's maxima
  const int n_alpha = early ? 1 : kAlphaSlots;
  float *top = early ? reinterpret_cast<float *>(ws + L.max_part) : nullptr;
  if (list == kListSelect) {
    // A: the transform, first pass: only the channel norms of X_wt leave the chip (the same
    // kernel clears the selection state)
    WCC_TRY(mark(WCC_T_HAAR_FWD, 0));
    if (src)
      WCC_TRY(launch_chain_norm(d, *src, wdw, L.G == 1 ? norm : part, top, L.G,
                                make_prep(ws, L, slots, quant ? alpha_in : 0.f), s));
    else
      WCC_TRY(launch_haar_norm(d, x, L.G == 1 ? norm : part, top, L.G,
                               make_prep(ws, L, slots, quant ? alpha_in : 0.f), wdw, s));
    WCC_TRY(mark(WCC_T_HAAR_FWD, 1));
    // B: norms, index set I (ascending), rank map for the inverse
    WCC_TRY(mark(WCC_T_NORM_SELECT, 0));
    WCC_TRY(launch_select(d, L.G == 1 ? norm : part, L.G, norm, k, ws, L, idx, jmap, top, tops, s));
    WCC_TRY(mark(WCC_T_NORM_SELECT, 1));
  } else {
    // a list that does not depend on the input: no norm pass, no selection
    WCC_TRY(mark(WCC_T_NORM_SELECT, 0));
    WCC_TRY(launch_alpha_init(slots, quant ? alpha_in : 0.f, s));
    if (list == kListPrefix)
      WCC_TRY(launch_jmap_prefix(d.B, (int64_t)d.H * d.W, k, jmap, idx_out, s));
    else
      WCC_TRY(launch_jmap_from_idx(idx_given, d.B, (int64_t)d.H * d.W, k, jmap, s));
    WCC_TRY(mark(WCC_T_NORM_SELECT, 1));
  }
  // A again + B': the transform, second pass: X_wt[I] is written straight into its compressed
  // place (the dropped coefficients never reach memory)
  WCC_TRY(mark(WCC_T_GATHER, 0));
  if (src)
    WCC_TRY(launch_chain_keep(d, k, *src, wdw, jmap, xc32, (quant && !given && !codes_now) ? slots : nullptr,
                              (given && codes_now) ? alpha_in : 0.f, early ? tops : nullptr, n_top,
                              early ? slots : nullptr, s));
  else
    WCC_TRY(launch_haar_keep(d, k, x, jmap, xc32, (quant && !given && !codes_now) ? slots : nullptr, wdw,
                             (given && codes_now) ? alpha_in : 0.f, early ? tops : nullptr, n_top,
                             early ? slots : nullptr, s));
  WCC_TRY(mark(WCC_T_GATHER, 1));
  // C: Y_wt = Conv(K_1x1, X_wt[I]) (kept coefficients still in fp32 are quantised as they are
  // loaded)
  WCC_TRY(mark(WCC_T_POINTWISE, 0));
  WCC_TRY(pointwise_any(ws, L, d, k, w, w_scale, xc32, !codes_now, slots, n_alpha,
                        quant ? alpha_out_dev : nullptr, yc, s));
  WCC_TRY(mark(WCC_T_POINTWISE, 1));
  if (stop_before_inverse) return WCC_OK;
  // D + E: Y^0[I] = Y_wt, inverse levels
  WCC_TRY(mark(WCC_T_SCATTER_IHAAR, 0));
  WCC_TRY(launch_scatter_ihaar(d, k, yc, jmap, y, reinterpret_cast<float *>(ws + L.scratch), residual, s));
  WCC_TRY(mark(WCC_T_SCATTER_IHAAR, 1));
  return WCC_OK;
}

// The two layers of the inverted residual block as layer descriptors.
wcc_status block_layers(const wcc_block_desc *bd, wcc_desc &d1, wcc_desc &d3) {
  if (!bd) return WCC_ERR_NULL;
  if (bd->C < 1 || bd->expansion < 1 || (int64_t)bd->C * bd->expansion > 65535) return WCC_ERR_SHAPE;
  d1 = wcc_desc{bd->B, bd->C, bd->C * bd->expansion, bd->H, bd->W, bd->levels, bd->keep_num,
                bd->keep_den, bd->w_dtype, bd->act_quant_bits, bd->act_dtype, bd->norm};
  d3 = d1;
  d3.C_in = d1.C_out;
  d3.C_out = bd->C;
  const wcc_status st = check_desc(&d1);
  return st != WCC_OK ? st : check_desc(&d3);
}

// What stands in front of the project layer's transform: K_dw's output in memory, K_dw folded
// into the passes that read the expand layer's output, or both rebuilt from the expand layer's
// compressed output (chained: possible when nobody asks for the middle tensors).
int block_front(const wcc_block_desc &bd, const wcc_desc &d3, bool wants_middle) {
  if (bd.W % 4 != 0) return kFrontNone;
  // Chained, a pass costs arithmetic and a gather per kept coefficient instead of bytes per
  // pixel: it wins while at most a third of the coefficients is kept (measured on the 256 x 256
  // block: 1.54 vs 1.93 ms at keep 1/8, 1.61 vs 2.25 ms at 1/4, 3.2 vs 2.8 ms at 1/2).
  const bool sparse = k_of(d3) * 3 <= (int64_t)d3.H * d3.W;
  return (!wants_middle && sparse && chain_supported(d3)) ? kFrontChain : kFrontDw;
}

struct BlockLayout { size_t t1, t2, layer1, layer3, total; };

// The two layers have workspaces of their own: chained, the project layer reads the expand
// layer's compressed output while it fills its own.
BlockLayout block_layout(const wcc_block_desc &bd, const wcc_desc &d1, const wcc_desc &d3) {
  BlockLayout L{};
  const size_t mid = align256((size_t)bd.B * d1.C_out * bd.H * bd.W * 4);
  L.t1 = 0;
  L.t2 = mid;
  L.layer1 = 2 * mid;
  L.layer3 = L.layer1 + ws_layout(d1).total;
  // (the chained front asks for the most channel groups, so its layout is the largest)
  const size_t b = std::max(ws_layout(d3, block_front(bd, d3, true)).total,
                            ws_layout(d3, block_front(bd, d3, false)).total);
  L.total = L.layer3 + b;
  return L;
}

}  // namespace wcc

using namespace wcc;

extern "C" {

const char *wcc_status_string(wcc_status s) {
  switch (s) {
    case WCC_OK: return "ok";
    case WCC_ERR_NULL: return "required pointer is NULL";
    case WCC_ERR_SHAPE: return "bad shape (sizes >= 1, levels in 1..4, H and W divisible by 2^levels)";
    case WCC_ERR_DTYPE: return "bad weight dtype or activation bit width";
    case WCC_ERR_KEEP: return "keep ratio does not give 1 <= k <= H*W";
    case WCC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case WCC_ERR_UNSUPPORTED: return "unsupported configuration";
    case WCC_ERR_HIP: return "HIP runtime error";
    case WCC_ERR_ALIGN: return "tensor pointer is not 16-byte aligned";
  }
  return "unknown status";
}

wcc_status wcc_create(wcc_ctx **out, int device) {
  if (!out) return WCC_ERR_NULL;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return WCC_ERR_HIP;
  // where this device keeps the static scratch array (asked with that device current)
  int prev = 0;
  void *sp = nullptr;
  if (hipGetDevice(&prev) != hipSuccess || hipSetDevice(device) != hipSuccess) return WCC_ERR_HIP;
  const hipError_t e = static_scratch_of(device, &sp);
  if (hipSetDevice(prev) != hipSuccess || e != hipSuccess) return WCC_ERR_HIP;
  wcc_ctx *c = new (std::nothrow) wcc_ctx;
  if (!c) return WCC_ERR_HIP;
  c->device = device;
  c->static_ws = sp;
  *out = c;
  return WCC_OK;
}

wcc_status wcc_destroy(wcc_ctx *ctx) {
  if (!ctx) return WCC_ERR_NULL;
  if (ctx->ev_ok)
    for (auto &p : ctx->ev) { (void)hipEventDestroy(p[0]); (void)hipEventDestroy(p[1]); }
  delete ctx;
  return WCC_OK;
}

wcc_status wcc_workspace_bytes(const wcc_desc *desc, size_t *bytes) {
  if (!bytes) return WCC_ERR_NULL;
  const wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  *bytes = ws_layout(*desc).total;
  return WCC_OK;
}

wcc_status wcc_set_workspace(wcc_ctx *ctx, void *dev_ptr, size_t bytes) {
  if (!ctx) return WCC_ERR_NULL;
  if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255)) return WCC_ERR_WORKSPACE;
  ctx->ws = dev_ptr;
  ctx->ws_bytes = dev_ptr ? bytes : 0;
  return WCC_OK;
}

int64_t wcc_k(const wcc_desc *desc) {
  if (check_desc(desc) != WCC_OK) return -1;
  return k_of(*desc);
}

wcc_status wcc_set_profiling(wcc_ctx *ctx, int enabled) {
  if (!ctx) return WCC_ERR_NULL;
  if (enabled && !ctx->ev_ok) {
    for (auto &p : ctx->ev)
      if (hipEventCreate(&p[0]) != hipSuccess || hipEventCreate(&p[1]) != hipSuccess) return WCC_ERR_HIP;
    ctx->ev_ok = true;
  }
  ctx->profiling = enabled != 0;
  ctx->have_times = false;
  for (bool &m : ctx->marked) m = false;
  return WCC_OK;
}

wcc_status wcc_stage_times(wcc_ctx *ctx, float *ms) {
  if (!ctx || !ms) return WCC_ERR_NULL;
  if (!ctx->have_times) return WCC_ERR_UNSUPPORTED;
  for (int i = 0; i < WCC_T_COUNT; ++i) {
    ms[i] = 0.f;
    if (!ctx->marked[i]) continue;  // a stage the last calls did not run
    if (hipEventSynchronize(ctx->ev[i][1]) != hipSuccess) return WCC_ERR_HIP;
    if (hipEventElapsedTime(&ms[i], ctx->ev[i][0], ctx->ev[i][1]) != hipSuccess) return WCC_ERR_HIP;
  }
  return WCC_OK;
}

wcc_status wcc_haar_fwd(wcc_ctx *ctx, const wcc_desc *desc, const float *x, float *coef,
                        float *norm, void *stream) {
  if (!ctx || !x || !coef) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (desc->act_dtype != WCC_F32) return WCC_ERR_UNSUPPORTED;  // fp32 feature maps only here
  if (misaligned(x) || misaligned(coef) || misaligned(norm)) return WCC_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const WsLayout L = ws_layout(*desc);
  const SelectPrep no_prep{nullptr, nullptr, 0.f};
  if (!norm || desc->norm == WCC_NORM_L2) {
    // (sums of squares are taken from the stored coefficients in a pass of their own)
    wcc_desc plain = *desc;
    plain.norm = WCC_NORM_L1;
    WCC_TRY(launch_haar_fwd(plain, x, coef, nullptr, L.G, no_prep, s));
    if (norm)
      WCC_TRY(launch_channel_norm(coef, desc->B, desc->C_in, (int64_t)desc->H * desc->W, true, norm, s));
    return WCC_OK;
  }
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  const int64_t BN = (int64_t)desc->B * desc->H * desc->W;
  if (L.G == 1) {
    WCC_TRY(launch_haar_fwd(*desc, x, coef, norm, 1, no_prep, s));
  } else {
    float *part = reinterpret_cast<float *>(static_cast<char *>(ctx->ws) + L.norm_part);
    WCC_TRY(launch_haar_fwd(*desc, x, coef, part, L.G, no_prep, s));
    WCC_TRY(launch_norm_reduce(part, L.G, BN, norm, s));
  }
  return WCC_OK;
}

wcc_status wcc_joint_topk(wcc_ctx *ctx, const wcc_desc *desc, const float *coef, const float *norm,
                          int32_t *idx, void *stream) {
  if (!ctx || !idx || (!coef && !norm)) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (misaligned(coef) || misaligned(norm) || misaligned(idx)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char *ws = static_cast<char *>(ctx->ws);
  if (!norm) {
    float *nw = reinterpret_cast<float *>(ws + L.norm);
    WCC_TRY(launch_channel_norm(coef, desc->B, desc->C_in, (int64_t)desc->H * desc->W,
                                desc->norm == WCC_NORM_L2, nw, s));
    norm = nw;
  }
  const int64_t k = k_of(*desc);
  WCC_TRY(launch_select_init(make_prep(ws, L, nullptr, 0.f), desc->B, s));
  WCC_TRY(launch_select(*desc, norm, 1, nullptr, k, ws, L, idx, nullptr, nullptr, nullptr, s));
  return WCC_OK;
}

wcc_status wcc_gather_quant(wcc_ctx *ctx, const wcc_desc *desc, const float *coef,
                            const int32_t *idx, float alpha_in, void *xc, float *alpha_dev,
                            void *stream) {
  if (!ctx || !coef || !idx || !xc) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  const bool quant = desc->act_quant_bits == 8;
  if (quant && !alpha_dev) return WCC_ERR_NULL;
  if (misaligned(coef) || misaligned(idx) || misaligned(xc)) return WCC_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t N = (int64_t)desc->H * desc->W, k = k_of(*desc);
  if (!quant) {
    WCC_TRY(launch_gather(coef, idx, desc->B, desc->C_in, N, k, static_cast<float *>(xc), nullptr, s));
    return WCC_OK;
  }
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  char *ws = static_cast<char *>(ctx->ws);
  float *xc32 = reinterpret_cast<float *>(ws + L.xc32);
  float *slots = reinterpret_cast<float *>(ws + L.alpha);
  WCC_TRY(launch_alpha_init(slots, alpha_in, s));
  WCC_TRY(launch_gather(coef, idx, desc->B, desc->C_in, N, k, xc32, alpha_in > 0.f ? nullptr : slots, s));
  WCC_TRY(launch_quantize(xc32, (int64_t)desc->B * desc->C_in * k, slots, alpha_dev,
                          static_cast<int8_t *>(xc), s));
  return WCC_OK;
}

wcc_status wcc_pointwise(wcc_ctx *ctx, const wcc_desc *desc, const void *w, const float *w_scale,
                         const void *xc, const float *alpha_dev, float *yc, void *stream) {
  if (!ctx || !w || !xc || !yc) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (coded(desc->w_dtype) && !w_scale) return WCC_ERR_NULL;
  if (desc->act_quant_bits == 8 && !alpha_dev) return WCC_ERR_NULL;
  if (misaligned(w) || misaligned(xc) || misaligned(yc)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if (desc->w_dtype == WCC_I4 && (st = need_ws(ctx, L)) != WCC_OK) return st;
  WCC_TRY(pointwise_any(static_cast<char *>(ctx->ws), L, *desc, k_of(*desc), w, w_scale, xc,
                        desc->act_quant_bits == 0, alpha_dev, 1, nullptr, yc,
                        static_cast<hipStream_t>(stream)));
  return WCC_OK;
}

wcc_status wcc_scatter_ihaar(wcc_ctx *ctx, const wcc_desc *desc, const float *yc,
                             const int32_t *idx, float *y, void *stream) {
  if (!ctx || !yc || !idx || !y) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (desc->act_dtype != WCC_F32) return WCC_ERR_UNSUPPORTED;  // fp32 feature maps only here
  if (misaligned(yc) || misaligned(idx) || misaligned(y)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t N = (int64_t)desc->H * desc->W, k = k_of(*desc);
  int32_t *jmap = reinterpret_cast<int32_t *>(static_cast<char *>(ctx->ws) + L.jmap);
  WCC_TRY(launch_jmap_from_idx(idx, desc->B, N, k, jmap, s));
  WCC_TRY(launch_scatter_ihaar(*desc, k, yc, jmap, y,
                               reinterpret_cast<float *>(static_cast<char *>(ctx->ws) + L.scratch),
                               nullptr, s));
  return WCC_OK;
}

wcc_status wcc_forward(wcc_ctx *ctx, const wcc_desc *desc, const void *x, const void *w,
                       const float *w_scale, float alpha_in, void *y, int32_t *idx_out,
                       float *alpha_out_dev, void *stream) {
  if (!ctx || !x || !w || !y) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (coded(desc->w_dtype) && !w_scale) return WCC_ERR_NULL;
  if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(idx_out)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool prof = ctx->profiling && ctx->ev_ok;
  st = forward_on(ctx, static_cast<char *>(ctx->ws), L, *desc, x, w, w_scale, alpha_in, y, idx_out,
                  alpha_out_dev, nullptr, nullptr, prof, s);
  if (st != WCC_OK) return st;
  if (prof) {
    WCC_TRY(hipEventRecord(ctx->ev[WCC_T_EVENT_PAIR][0], s));
    WCC_TRY(hipEventRecord(ctx->ev[WCC_T_EVENT_PAIR][1], s));
    ctx->marked[WCC_T_EVENT_PAIR] = true;
    ctx->have_times = true;
  }
  return WCC_OK;
}

wcc_status wcc_forward_static(wcc_ctx *ctx, const wcc_desc *desc, const void *x, const void *w,
                              const float *w_scale, float alpha_in, void *y, int32_t *idx_out,
                              float *alpha_out_dev, void *stream) {
  if (!ctx || !x || !w || !y) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (coded(desc->w_dtype) && !w_scale) return WCC_ERR_NULL;
  if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(idx_out)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if (L.total > (size_t)WCC_STATIC_SCRATCH_BYTES) return WCC_ERR_WORKSPACE;
  // the scratch array belongs to the context's device: the kernels must run there
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) return WCC_ERR_HIP;
  if (cur != ctx->device || ctx->static_ws == nullptr) return WCC_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // every buffer that has to start at a known value (histograms, alpha slots) is cleared by the
  // first kernel of the layer itself, as with a caller's workspace of unknown content
  return forward_on(ctx, static_cast<char *>(ctx->static_ws), L, *desc, x, w, w_scale, alpha_in, y,
                    idx_out, alpha_out_dev, nullptr, nullptr, false, s);
}

wcc_status wcc_forward_fixed(wcc_ctx *ctx, const wcc_desc *desc, const void *x, const void *w,
                             const float *w_scale, float alpha_in, const int32_t *idx, void *y,
                             float *alpha_out_dev, void *stream) {
  if (!ctx || !x || !w || !y) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (coded(desc->w_dtype) && !w_scale) return WCC_ERR_NULL;
  if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(idx)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool prof = ctx->profiling && ctx->ev_ok;
  st = forward_on(ctx, static_cast<char *>(ctx->ws), L, *desc, x, w, w_scale, alpha_in, y, nullptr,
                  alpha_out_dev, nullptr, nullptr, prof, s, idx ? kListGiven : kListPrefix, idx);
  if (st != WCC_OK) return st;
  if (prof) {
    WCC_TRY(hipEventRecord(ctx->ev[WCC_T_EVENT_PAIR][0], s));
    WCC_TRY(hipEventRecord(ctx->ev[WCC_T_EVENT_PAIR][1], s));
    ctx->marked[WCC_T_EVENT_PAIR] = true;
    ctx->have_times = true;
  }
  return WCC_OK;
}

wcc_status wcc_block_workspace_bytes(const wcc_block_desc *desc, size_t *bytes) {
  if (!bytes) return WCC_ERR_NULL;
  wcc_desc d1, d3;
  const wcc_status st = block_layers(desc, d1, d3);
  if (st != WCC_OK) return st;
  *bytes = block_layout(*desc, d1, d3).total;
  return WCC_OK;
}

int32_t wcc_block_is_chained(const wcc_block_desc *desc) {
  wcc_desc d1, d3;
  if (block_layers(desc, d1, d3) != WCC_OK) return -1;
  return block_front(*desc, d3, false) == kFrontChain ? 1 : 0;
}

wcc_status wcc_depthwise3x3(wcc_ctx *ctx, int32_t B, int32_t C, int32_t H, int32_t W,
                            const float *x, const float *w, float *y, void *stream) {
  if (!ctx || !x || !w || !y) return WCC_ERR_NULL;
  if (B < 1 || C < 1 || H < 1 || W < 1 || B > 65535 || C > 65535) return WCC_ERR_SHAPE;
  if ((int64_t)H * W > ((int64_t)1 << 30)) return WCC_ERR_SHAPE;
  if (misaligned(x) || misaligned(y)) return WCC_ERR_ALIGN;
  WCC_TRY(launch_depthwise3x3(B, C, H, W, x, w, y, static_cast<hipStream_t>(stream)));
  return WCC_OK;
}

wcc_status wcc_set_block_profile_layer(wcc_ctx *ctx, int layer) {
  if (!ctx) return WCC_ERR_NULL;
  if (layer != 0 && layer != 1) return WCC_ERR_SHAPE;
  ctx->block_profile_layer = layer;
  return WCC_OK;
}

wcc_status wcc_block_forward(wcc_ctx *ctx, const wcc_block_desc *desc, const void *x,
                             const void *w1, const float *w1_scale, const float *w_dw,
                             const void *w3, const float *w3_scale, void *y, void *t1_out,
                             float *t2_out, int32_t *idx1_out, int32_t *idx3_out, void *stream) {
  if (!ctx || !x || !w1 || !w_dw || !w3 || !y) return WCC_ERR_NULL;
  wcc_desc d1, d3;
  wcc_status st = block_layers(desc, d1, d3);
  if (st != WCC_OK) return st;
  if (coded(desc->w_dtype) && (!w1_scale || !w3_scale)) return WCC_ERR_NULL;
  if (misaligned(x) || misaligned(w1) || misaligned(w3) || misaligned(y) || misaligned(t1_out) ||
      misaligned(t2_out) || misaligned(idx1_out) || misaligned(idx3_out))
    return WCC_ERR_ALIGN;
  // K_dw is folded into the two transform passes of the project layer (its output is never
  // written) when the width allows; the stand-alone kernel runs otherwise, and when the caller
  // asks for K_dw's output.  It reads and writes fp32 only.
  const bool fold = desc->W % 4 == 0;
  if (desc->act_dtype != WCC_F32 && (!fold || t2_out)) return WCC_ERR_UNSUPPORTED;
  const BlockLayout BL = block_layout(*desc, d1, d3);
  if (!ctx->ws || ctx->ws_bytes < BL.total) return WCC_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char *ws = static_cast<char *>(ctx->ws);
  const bool prof = ctx->profiling && ctx->ev_ok;
  const int front = block_front(*desc, d3, t1_out != nullptr || t2_out != nullptr);
  const WsLayout L1 = ws_layout(d1), L3 = ws_layout(d3, front);

  if (front == kFrontChain) {
    // Chained: the expand layer stops at its compressed output; the project layer's transform
    // passes rebuild the rows they need from it, convolve and transform them.  Neither middle
    // tensor exists.
    st = forward_on(ctx, ws + BL.layer1, L1, d1, x, w1, w1_scale, 0.f, nullptr, idx1_out, nullptr,
                    nullptr, nullptr, prof && ctx->block_profile_layer == 0, s, kListSelect, nullptr,
                    nullptr, true);
    if (st != WCC_OK) return st;
    const ChainSrc src{reinterpret_cast<const float *>(ws + BL.layer1 + L1.yc),
                       reinterpret_cast<const int32_t *>(ws + BL.layer1 + L1.jmap), k_of(d1)};
    st = forward_on(ctx, ws + BL.layer3, L3, d3, nullptr, w3, w3_scale, 0.f, y, idx3_out, nullptr, x,
                    w_dw, prof && ctx->block_profile_layer == 1, s, kListSelect, nullptr, &src);
    if (st != WCC_OK) return st;
  } else {
    void *t1 = t1_out ? t1_out : static_cast<void *>(ws + BL.t1);
    float *t2 = t2_out ? t2_out : reinterpret_cast<float *>(ws + BL.t2);
    // K1 (expand), K_dw, K3 (project) with the skip connection added by the last kernel
    st = forward_on(ctx, ws + BL.layer1, L1, d1, x, w1, w1_scale, 0.f, t1, idx1_out, nullptr,
                    nullptr, nullptr, prof && ctx->block_profile_layer == 0, s);
    if (st != WCC_OK) return st;
    if (!fold || t2_out) {
      if (prof) WCC_TRY(hipEventRecord(ctx->ev[WCC_T_DEPTHWISE][0], s));
      WCC_TRY(launch_depthwise3x3(d3.B, d3.C_in, d3.H, d3.W, static_cast<const float *>(t1), w_dw, t2, s));
      if (prof) {
        WCC_TRY(hipEventRecord(ctx->ev[WCC_T_DEPTHWISE][1], s));
        ctx->marked[WCC_T_DEPTHWISE] = true;
      }
    }
    st = forward_on(ctx, ws + BL.layer3, L3, d3, fold ? t1 : static_cast<void *>(t2), w3, w3_scale, 0.f, y,
                    idx3_out, nullptr, x, fold ? w_dw : nullptr,
                    prof && ctx->block_profile_layer == 1, s);
    if (st != WCC_OK) return st;
  }
  if (prof) {
    WCC_TRY(hipEventRecord(ctx->ev[WCC_T_EVENT_PAIR][0], s));
    WCC_TRY(hipEventRecord(ctx->ev[WCC_T_EVENT_PAIR][1], s));
    ctx->marked[WCC_T_EVENT_PAIR] = true;
    ctx->have_times = true;
  }
  return WCC_OK;
}

}  // extern "C"
