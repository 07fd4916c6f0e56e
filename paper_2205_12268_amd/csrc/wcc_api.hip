// C ABI of libwcc: argument checks, workspace carving, and the order in which the kernels of
// Alg. 1 are enqueued.  No arithmetic of the method happens on the host.
#include <new>

#include "wcc_internal.h"

struct wcc_ctx {
  int device = 0;
  void *ws = nullptr;
  size_t ws_bytes = 0;
  bool profiling = false;
  bool have_times = false;
  hipEvent_t ev[WCC_T_COUNT][2] = {};
  bool ev_ok = false;
};

namespace wcc {
namespace {

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

wcc_status check_desc(const wcc_desc *d) {
  if (!d) return WCC_ERR_NULL;
  if (d->B < 1 || d->C_in < 1 || d->C_out < 1 || d->H < 2 || d->W < 2) return WCC_ERR_SHAPE;
  if (d->levels < 1 || d->levels > kMaxLevels) return WCC_ERR_SHAPE;
  const int s = 1 << d->levels;
  if (d->H % s || d->W % s) return WCC_ERR_SHAPE;
  // grid limits and 32-bit in-plane offsets
  if (d->B > 65535 || d->C_in > 65535 || d->C_out > 65535) return WCC_ERR_SHAPE;
  if ((int64_t)d->H * d->W > ((int64_t)1 << 30)) return WCC_ERR_SHAPE;
  if (d->w_dtype != WCC_F32 && d->w_dtype != WCC_BF16 && d->w_dtype != WCC_I8) return WCC_ERR_DTYPE;
  if (d->act_quant_bits != 0 && d->act_quant_bits != 8) return WCC_ERR_DTYPE;
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

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

wcc_status need_ws(const wcc_ctx *ctx, const WsLayout &L) {
  if (!ctx->ws || ctx->ws_bytes < L.total) return WCC_ERR_WORKSPACE;
  return WCC_OK;
}

}  // namespace

WsLayout ws_layout(const wcc_desc &d) {
  WsLayout L{};
  const size_t N = (size_t)d.H * d.W, B = d.B, k = (size_t)k_of(d);
  L.G = forward_groups(d);
  L.nblk = (int)((N + kSelectChunk - 1) / kSelectChunk);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  L.norm_part = take((size_t)L.G * B * N * 4);
  L.norm = take(B * N * 4);
  L.hist = take(B * 3 * kRadixBins * 4);
  L.state = take(B * sizeof(SelectState));
  L.block_sfx = take(B * (size_t)L.nblk * kSfxStride * 2);
  L.block_gthi = take(B * (size_t)L.nblk * 4);
  L.jmap = take(B * N * 4);
  L.idx = take(B * k * 4);
  L.alpha = take(256);
  L.scratch = take(kInvScratchBytes);
  L.xc32 = take(B * (size_t)d.C_in * k * 4);
  L.yc = take(B * (size_t)d.C_out * k * 4);
  L.total = off;
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
  wcc_ctx *c = new (std::nothrow) wcc_ctx;
  if (!c) return WCC_ERR_HIP;
  c->device = device;
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
  return WCC_OK;
}

wcc_status wcc_stage_times(wcc_ctx *ctx, float *ms) {
  if (!ctx || !ms) return WCC_ERR_NULL;
  if (!ctx->have_times) return WCC_ERR_UNSUPPORTED;
  for (int i = 0; i < WCC_T_COUNT; ++i) {
    if (hipEventSynchronize(ctx->ev[i][1]) != hipSuccess) return WCC_ERR_HIP;
    if (hipEventElapsedTime(&ms[i], ctx->ev[i][0], ctx->ev[i][1]) != hipSuccess) return WCC_ERR_HIP;
  }
  return WCC_OK;
}

#define WCC_TRY(expr)                                 \
  do {                                                \
    if ((expr) != hipSuccess) return WCC_ERR_HIP;     \
  } while (0)

wcc_status wcc_haar_fwd(wcc_ctx *ctx, const wcc_desc *desc, const float *x, float *coef,
                        float *norm, void *stream) {
  if (!ctx || !x || !coef) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (misaligned(x) || misaligned(coef) || misaligned(norm)) return WCC_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const WsLayout L = ws_layout(*desc);
  const SelectPrep no_prep{nullptr, nullptr, 0.f};
  if (!norm) {
    WCC_TRY(launch_haar_fwd(*desc, x, coef, nullptr, L.G, no_prep, s));
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
    WCC_TRY(launch_channel_norm(coef, desc->B, desc->C_in, (int64_t)desc->H * desc->W, nw, s));
    norm = nw;
  }
  const int64_t k = k_of(*desc);
  WCC_TRY(launch_select_init(make_prep(ws, L, nullptr, 0.f), desc->B, s));
  WCC_TRY(launch_select(*desc, norm, 1, nullptr, k, ws, L, idx, nullptr, s));
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
  if (desc->w_dtype == WCC_I8 && !w_scale) return WCC_ERR_NULL;
  if (desc->act_quant_bits == 8 && !alpha_dev) return WCC_ERR_NULL;
  if (misaligned(w) || misaligned(xc) || misaligned(yc)) return WCC_ERR_ALIGN;
  WCC_TRY(launch_pointwise(*desc, k_of(*desc), w, w_scale, xc, desc->act_quant_bits == 0, alpha_dev,
                           false, nullptr, yc, static_cast<hipStream_t>(stream)));
  return WCC_OK;
}

wcc_status wcc_scatter_ihaar(wcc_ctx *ctx, const wcc_desc *desc, const float *yc,
                             const int32_t *idx, float *y, void *stream) {
  if (!ctx || !yc || !idx || !y) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (misaligned(yc) || misaligned(idx) || misaligned(y)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t N = (int64_t)desc->H * desc->W, k = k_of(*desc);
  int32_t *jmap = reinterpret_cast<int32_t *>(static_cast<char *>(ctx->ws) + L.jmap);
  WCC_TRY(launch_jmap_from_idx(idx, desc->B, N, k, jmap, s));
  WCC_TRY(launch_scatter_ihaar(*desc, k, yc, jmap, y,
                               reinterpret_cast<float *>(static_cast<char *>(ctx->ws) + L.scratch), s));
  return WCC_OK;
}

wcc_status wcc_forward(wcc_ctx *ctx, const wcc_desc *desc, const float *x, const void *w,
                       const float *w_scale, float alpha_in, float *y, int32_t *idx_out,
                       float *alpha_out_dev, void *stream) {
  if (!ctx || !x || !w || !y) return WCC_ERR_NULL;
  wcc_status st = check_desc(desc);
  if (st != WCC_OK) return st;
  if (desc->w_dtype == WCC_I8 && !w_scale) return WCC_ERR_NULL;
  if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(idx_out)) return WCC_ERR_ALIGN;
  const WsLayout L = ws_layout(*desc);
  if ((st = need_ws(ctx, L)) != WCC_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char *ws = static_cast<char *>(ctx->ws);
  const wcc_desc &d = *desc;
  const int64_t k = k_of(d);
  const bool quant = d.act_quant_bits == 8;

  float *part = reinterpret_cast<float *>(ws + L.norm_part);
  float *norm = reinterpret_cast<float *>(ws + L.norm);
  int32_t *jmap = reinterpret_cast<int32_t *>(ws + L.jmap);
  int32_t *idx = idx_out ? idx_out : reinterpret_cast<int32_t *>(ws + L.idx);
  float *slots = reinterpret_cast<float *>(ws + L.alpha);
  float *xc32 = reinterpret_cast<float *>(ws + L.xc32);
  float *yc = reinterpret_cast<float *>(ws + L.yc);

  const bool prof = ctx->profiling && ctx->ev_ok;
  auto mark = [&](int stage, int which) -> hipError_t {
    return prof ? hipEventRecord(ctx->ev[stage][which], s) : hipSuccess;
  };

  // A: the transform, first pass: only the channel norms of X_wt leave the chip (the same
  // kernel clears the selection state)
  WCC_TRY(mark(WCC_T_HAAR_FWD, 0));
  WCC_TRY(launch_haar_norm(d, x, L.G == 1 ? norm : part, L.G,
                           make_prep(ws, L, slots, quant ? alpha_in : 0.f), s));
  WCC_TRY(mark(WCC_T_HAAR_FWD, 1));
  // B: norms, index set I (ascending), rank map for the inverse
  WCC_TRY(mark(WCC_T_NORM_SELECT, 0));
  WCC_TRY(launch_select(d, L.G == 1 ? norm : part, L.G, norm, k, ws, L, idx, jmap, s));
  WCC_TRY(mark(WCC_T_NORM_SELECT, 1));
  // A again + B': the transform, second pass: X_wt[I] is written straight into its compressed
  // place (the dropped coefficients never reach memory); alpha = max |kept coefficient|
  WCC_TRY(mark(WCC_T_GATHER, 0));
  WCC_TRY(launch_haar_keep(d, k, x, jmap, xc32, (quant && !(alpha_in > 0.f)) ? slots : nullptr, s));
  WCC_TRY(mark(WCC_T_GATHER, 1));
  // C: Y_wt = Conv(K_1x1, X_wt[I]); the kept coefficients are quantised as they are loaded
  WCC_TRY(mark(WCC_T_POINTWISE, 0));
  WCC_TRY(launch_pointwise(d, k, w, w_scale, xc32, true, slots, true, quant ? alpha_out_dev : nullptr,
                           yc, s));
  WCC_TRY(mark(WCC_T_POINTWISE, 1));
  // D + E: Y^0[I] = Y_wt, inverse levels
  WCC_TRY(mark(WCC_T_SCATTER_IHAAR, 0));
  WCC_TRY(launch_scatter_ihaar(d, k, yc, jmap, y, reinterpret_cast<float *>(ws + L.scratch), s));
  WCC_TRY(mark(WCC_T_SCATTER_IHAAR, 1));
  WCC_TRY(mark(WCC_T_EVENT_PAIR, 0));
  WCC_TRY(mark(WCC_T_EVENT_PAIR, 1));
  if (prof) ctx->have_times = true;
  return WCC_OK;
}

}  // extern "C"
