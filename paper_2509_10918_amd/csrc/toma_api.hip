// C-ABI entry points of libtoma: argument checks on the host, workspace layout, stage launches.
#include <math.h>

#include <algorithm>
#include <mutex>

#include "toma_internal.h"

namespace toma {

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

int make_shape(const toma_desc *d, const toma_attn_desc *a, Shape *s) {
  if (!d) return TOMA_ERR_NULL;
  if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->tile_h <= 0 || d->tile_w <= 0 || d->d_loc <= 0)
    return TOMA_ERR_SHAPE;
  if (d->H % d->tile_h || d->W % d->tile_w) return TOMA_ERR_SHAPE;
  if (!(d->tau > 0.0f) || !isfinite(d->tau) || !isfinite(d->logit_scale) || d->logit_scale < 0.0f)
    return TOMA_ERR_SHAPE;
  if (d->dtype != TOMA_F32 && d->dtype != TOMA_BF16) return TOMA_ERR_UNSUPPORTED;
  s->B = d->B; s->H = d->H; s->W = d->W; s->C = d->C;
  s->tile_h = d->tile_h; s->tile_w = d->tile_w; s->d_loc = d->d_loc;
  s->N = d->H * d->W;
  s->P = (d->H / d->tile_h) * (d->W / d->tile_w);
  s->n_loc = d->tile_h * d->tile_w;
  if (d->d_loc > s->n_loc) return TOMA_ERR_SHAPE;
  if (d->merge_regions != 1 && d->merge_regions != s->P) return TOMA_ERR_SHAPE;
  if (d->C % 32) return TOMA_ERR_UNSUPPORTED;
  if (s->n_loc % 16 || s->n_loc > 2048) return TOMA_ERR_UNSUPPORTED;  // (the selection kernels' largest region)
  // kernels index inside one sample with 32-bit element offsets and launch one thread per element
  // of a tensor in places: a sample's tokens must stay below 2^31 elements, the batch below 2^38
  if ((long long)s->N * d->C >= (1ll << 31) || (long long)d->B * s->N * d->C >= (1ll << 38)) return TOMA_ERR_UNSUPPORTED;
  s->R = d->merge_regions;
  s->D = s->P * d->d_loc;
  s->Nr = s->N / s->R;
  s->Dr = s->D / s->R;
  s->scale = d->logit_scale > 0.0f ? d->logit_scale : 1.0f / d->tau;
  s->dtype = d->dtype;
  s->heads = s->head_dim = s->T = s->L = 0;
  if (a) {
    if (a->heads <= 0 || a->head_dim <= 0 || a->t_extra < 0) return TOMA_ERR_SHAPE;
    if ((long long)a->heads * a->head_dim != d->C) return TOMA_ERR_SHAPE;
    if (a->head_dim != 32 && a->head_dim != 64 && a->head_dim != 128) return TOMA_ERR_UNSUPPORTED;
    s->heads = a->heads; s->head_dim = a->head_dim; s->T = a->t_extra; s->L = s->D + a->t_extra;
    if ((long long)s->L * d->C >= (1ll << 31) || (long long)d->B * s->L * d->C >= (1ll << 38)) return TOMA_ERR_UNSUPPORTED;
  }
  return TOMA_OK;
}

void plan_workspace(const Shape &s, Workspace *w) {
  size_t es = s.dtype == TOMA_BF16 ? 2 : 4;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
  // row strides of the partial-result arrays: one entry per wave slice of the weights product
  // (sources x destinations x C), whose block tile is planned here exactly as at launch
  // (the statistics pass always gets its room: the single-pass weights kernel does not use it, the
  // entry points that recompute weights instead of storing them do)
  if (gemm_async_fits(s.Nr, s.Dr, s.C, (int)es)) {
    const GemmPlan pw = plan_gemm_async(s.Nr, s.Dr, s.C, s.B * s.R, (int)es, false, false, false, 3);
    w->stat_parts = 2 * ((s.Dr + pw.bn - 1) / pw.bn);
    w->z_parts = 4 * ((s.Nr + pw.bm - 1) / pw.bm);
  } else {
    w->stat_parts = 2 * ((s.Dr + 63) / 64);
    w->z_parts = 2 * ((s.Nr + 63) / 64);
  }
  if (weights_single_pass(s.Nr, s.Dr, s.C, s.B * s.R, (int)es)) w->z_parts = s.Nr / 32;  // one partial row sum per 32-source workgroup
  w->sim = take((size_t)s.B * s.P * s.n_loc * s.n_loc * sizeof(float));
  w->gram = take(gram_i8_workspace_bytes(s));  // limb planes, norms and flags of the int8 similarity kernel
  w->stats = take((size_t)s.B * s.N * w->stat_parts * 2 * sizeof(float));
  w->lse = take((size_t)s.B * s.N * sizeof(float));
  w->zpart = take((size_t)s.B * s.D * w->z_parts * sizeof(float));
  w->os = take((size_t)s.B * s.D * s.C * es);
  size_t qkv = (size_t)s.B * s.L * s.C * es;
  w->q = take(qkv); w->k = take(qkv); w->v = take(qkv); w->oh = take(qkv);
  w->xm = take((size_t)s.B * s.D * s.C * es);  // merged tokens and attention output of toma_layer
  w->o = take(qkv);
  // fp32 partial tiles of the merge / unmerge products when their K is split between workgroups
  size_t part = 0;
  if (gemm_async_fits(s.Dr, s.C, s.Nr, (int)es)) {
    const GemmPlan pm = plan_gemm_async(s.Dr, s.C, s.Nr, s.B * s.R, (int)es, true, false, true, 1);
    if (pm.nsplit > 1) part = (size_t)pm.nsplit * s.B * s.D * s.C * sizeof(float);
  }
  if (gemm_async_fits(s.Nr, s.C, s.Dr, (int)es)) {
    const GemmPlan pu = plan_gemm_async(s.Nr, s.C, s.Dr, s.B * s.R, (int)es, true, true, true, 1);
    if (pu.nsplit > 1) part = std::max(part, (size_t)pu.nsplit * s.B * s.N * s.C * sizeof(float));
  }
  w->split = take(part);
  w->pinv = take(pinv_workspace_bytes(s));
  w->fcache = take(fused_cache_bytes(s, *w));  // statistics of recomputed weights inside one toma_layer call  // eigenvectors and G^+ of the Moore-Penrose unmerge
  // the occupancy map of A is not scratch: it belongs to the caller's cache, next to (A, Z)
  if (occupancy_pays(s.Nr, s.Dr, s.C, (int)es)) {
    w->occ_db = (s.Dr + kOccDest - 1) / kOccDest;
    w->occ_sb = s.Nr / kOccSrc;
    w->occ_bytes = up256((size_t)s.B * s.R * w->occ_db * w->occ_sb);
  } else {
    w->occ_db = w->occ_sb = 0;
    w->occ_bytes = 0;
  }
  // Z from the merge product's own A fragments: wherever that product keeps K whole in every workgroup
  // (planned here exactly as at launch)
  w->z_in_merge = gemm_async_fits(s.Dr, s.C, s.Nr, (int)es) &&
                  plan_map_product(s.Dr, s.C, s.Nr, s.B * s.R, (int)es, false, true, w->occ_sb != 0).nsplit == 1;
  w->total = off;
}

static bool misaligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

// Shared prologue of every call: shape, workspace size and alignment.
static int prepare(const toma_desc *d, const toma_attn_desc *a, void *ws, size_t ws_bytes, Shape *s, Workspace *w) {
  int rc = make_shape(d, a, s);
  if (rc != TOMA_OK) return rc;
  plan_workspace(*s, w);
  if (!ws) return TOMA_ERR_NULL;
  if (misaligned(ws, 256)) return TOMA_ERR_ALIGN;
  if (ws_bytes < w->total) return TOMA_ERR_WORKSPACE;
  return TOMA_OK;
}

}  // namespace toma

using namespace toma;

#define TOMA_API extern "C" __attribute__((visibility("default")))

TOMA_API size_t toma_workspace_bytes(const toma_desc *desc, const toma_attn_desc *attn) {
  Shape s;
  Workspace w;
  if (make_shape(desc, attn, &s) != TOMA_OK) return 0;
  plan_workspace(s, &w);
  return w.total;
}

TOMA_API const char *toma_status_string(int status) {
  switch (status) {
    case TOMA_OK: return "ok";
    case TOMA_ERR_NULL: return "null pointer";
    case TOMA_ERR_SHAPE: return "invalid shape";
    case TOMA_ERR_ALIGN: return "misaligned pointer";
    case TOMA_ERR_WORKSPACE: return "workspace too small";
    case TOMA_ERR_UNSUPPORTED: return "unsupported configuration";
    case TOMA_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

TOMA_API int toma_select(const toma_desc *desc, const void *X, int32_t *idx, float *gain_opt, float *gap_opt,
                         void *ws, size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!X || !idx) return TOMA_ERR_NULL;
  if (misaligned(X, 16) || misaligned(idx, 4) || (gain_opt && misaligned(gain_opt, 4)) ||
      (gap_opt && misaligned(gap_opt, 4)))
    return TOMA_ERR_ALIGN;
  return launch_select(s, X, idx, gain_opt, gap_opt, static_cast<char *>(ws), w, static_cast<hipStream_t>(stream));
}

// The block map travels with (A, Z): required exactly when the shape uses one.
static int check_map(const Workspace &w, const void *amap) {
  if (w.occ_bytes != 0 && !amap) return TOMA_ERR_NULL;
  if (amap && misaligned(amap, 16)) return TOMA_ERR_ALIGN;
  return TOMA_OK;
}

TOMA_API size_t toma_map_bytes(const toma_desc *desc) {
  Shape s;
  Workspace w;
  if (make_shape(desc, nullptr, &s) != TOMA_OK) return 0;
  plan_workspace(s, &w);
  return w.occ_bytes;
}

TOMA_API int toma_map_build(const toma_desc *desc, const void *A, void *amap, void *stream) {
  Shape s; Workspace w;
  int rc = make_shape(desc, nullptr, &s);
  if (rc != TOMA_OK) return rc;
  plan_workspace(s, &w);
  if (!A) return TOMA_ERR_NULL;
  if (misaligned(A, 16)) return TOMA_ERR_ALIGN;
  rc = check_map(w, amap);
  if (rc != TOMA_OK) return rc;
  return launch_occupancy(s, A, static_cast<uint8_t *>(amap), w, static_cast<hipStream_t>(stream));
}

// ---- selection without a caller workspace ------------------------------------------------------
// The selection's scratch (the regions' similarity matrices) in a buffer the library owns: a
// file-scope device array, present once on every GPU the library's code is loaded on.  In host code
// the array's name is only a handle; its device address on the current GPU comes from
// hipGetSymbolAddress, asked once per device and kept.
static __device__ __align__(256) unsigned char scratch[TOMA_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];

static int static_scratch(char **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TOMA_ERR_LAUNCH;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return TOMA_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<char *>(g_scratch_ptr[dev]);
  return TOMA_OK;
}

TOMA_API int toma_select_static(const toma_desc *desc, const void *X, int32_t *idx, float *gain_opt, float *gap_opt,
                                void *stream) {
  Shape s; Workspace w;
  int rc = make_shape(desc, nullptr, &s);
  if (rc != TOMA_OK) return rc;
  if (!X || !idx) return TOMA_ERR_NULL;
  if (misaligned(X, 16) || misaligned(idx, 4) || (gain_opt && misaligned(gain_opt, 4)) ||
      (gap_opt && misaligned(gap_opt, 4)))
    return TOMA_ERR_ALIGN;
  // the selection uses only the similarity sections of the workspace: they come first in its layout
  plan_workspace(s, &w);
  const size_t need = w.gram + up256(gram_i8_workspace_bytes(s));
  if (w.sim != 0 || need > (size_t)TOMA_STATIC_SCRATCH_BYTES) return TOMA_ERR_WORKSPACE;
  char *buf = nullptr;
  rc = static_scratch(&buf);
  if (rc != TOMA_OK) return rc;
  return launch_select(s, X, idx, gain_opt, gap_opt, buf, w, static_cast<hipStream_t>(stream));
}

TOMA_API int toma_merge(const toma_desc *desc, const void *X, const int32_t *idx, void *A, float *Z, void *amap,
                        void *Xm, void *ws, size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!X || !idx || !A || !Z || !Xm) return TOMA_ERR_NULL;
  if (misaligned(X, 16) || misaligned(A, 16) || misaligned(Xm, 16) || misaligned(Z, 4) || misaligned(idx, 4))
    return TOMA_ERR_ALIGN;
  rc = check_map(w, amap);
  if (rc != TOMA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t *occ = static_cast<uint8_t *>(amap);
  rc = launch_weights(s, X, idx, A, Z, occ, static_cast<char *>(ws), w, st);
  if (rc != TOMA_OK) return rc;
  return launch_merge(s, X, A, Z, true, occ, Xm, static_cast<char *>(ws), w, st);
}

TOMA_API int toma_merge_cached(const toma_desc *desc, const void *X, const void *A, const float *Z,
                               const void *amap, void *Xm, void *ws, size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!X || !A || !Z || !Xm) return TOMA_ERR_NULL;
  if (misaligned(X, 16) || misaligned(A, 16) || misaligned(Xm, 16) || misaligned(Z, 4)) return TOMA_ERR_ALIGN;
  rc = check_map(w, amap);
  if (rc != TOMA_OK) return rc;
  return launch_merge(s, X, A, const_cast<float *>(Z), false, static_cast<const uint8_t *>(amap), Xm, static_cast<char *>(ws), w,
                      static_cast<hipStream_t>(stream));
}

TOMA_API int toma_attend(const toma_desc *desc, const toma_attn_desc *attn, const void *Xm,
                         const void *X_extra_opt, const void *Wq, const void *Wk, const void *Wv,
                         const void *Wo_opt, void *O, void *ws, size_t ws_bytes, void *stream) {
  if (!attn) return TOMA_ERR_NULL;
  Shape s; Workspace w;
  int rc = prepare(desc, attn, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!Xm || !Wq || !Wk || !Wv || !O) return TOMA_ERR_NULL;
  if ((s.T > 0) != (X_extra_opt != nullptr)) return TOMA_ERR_NULL;
  if (misaligned(Xm, 16) || misaligned(Wq, 16) || misaligned(Wk, 16) || misaligned(Wv, 16) || misaligned(O, 16) ||
      (X_extra_opt && misaligned(X_extra_opt, 16)) || (Wo_opt && misaligned(Wo_opt, 16)))
    return TOMA_ERR_ALIGN;
  return launch_attend(s, Xm, X_extra_opt, Wq, Wk, Wv, Wo_opt, O, nullptr, nullptr, static_cast<char *>(ws), w,
                       static_cast<hipStream_t>(stream));
}

TOMA_API int toma_cross_attend(const toma_desc *desc, const toma_attn_desc *attn, const void *U, const void *Ctx,
                               int32_t t_ctx, int32_t c_ctx, const void *Wq, const void *Wk, const void *Wv,
                               const void *Wo_opt, void *O, void *ws, size_t ws_bytes, void *stream) {
  if (!attn) return TOMA_ERR_NULL;
  Shape s; Workspace w;
  int rc = prepare(desc, attn, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (t_ctx <= 0 || c_ctx <= 0) return TOMA_ERR_SHAPE;
  // keys and values of the context share the workspace sections sized for the L query rows
  if (c_ctx % 32 || t_ctx > s.L || (long long)t_ctx * c_ctx >= (1ll << 31)) return TOMA_ERR_UNSUPPORTED;
  if (!U || !Ctx || !Wq || !Wk || !Wv || !O) return TOMA_ERR_NULL;
  if (misaligned(U, 16) || misaligned(Ctx, 16) || misaligned(Wq, 16) || misaligned(Wk, 16) || misaligned(Wv, 16) ||
      misaligned(O, 16) || (Wo_opt && misaligned(Wo_opt, 16)))
    return TOMA_ERR_ALIGN;
  return launch_cross_attend(s, U, Ctx, t_ctx, c_ctx, Wq, Wk, Wv, Wo_opt, O, static_cast<char *>(ws), w,
                             static_cast<hipStream_t>(stream));
}

TOMA_API int toma_unmerge(const toma_desc *desc, const void *A, const float *Z, const void *amap, const void *O,
                          int32_t o_rows, void *Y, void *ws, size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!A || !Z || !O || !Y) return TOMA_ERR_NULL;
  if (o_rows < s.D) return TOMA_ERR_SHAPE;
  if (misaligned(A, 16) || misaligned(O, 16) || misaligned(Y, 16) || misaligned(Z, 4)) return TOMA_ERR_ALIGN;
  rc = check_map(w, amap);
  if (rc != TOMA_OK) return rc;
  return launch_unmerge(s, A, Z, static_cast<const uint8_t *>(amap), O, o_rows, false, Y, static_cast<char *>(ws), w,
                        static_cast<hipStream_t>(stream));
}

TOMA_API size_t toma_recompute_cache_bytes(const toma_desc *desc) {
  Shape s;
  Workspace w;
  if (make_shape(desc, nullptr, &s) != TOMA_OK) return 0;
  plan_workspace(s, &w);
  return fused_cache_bytes(s, w);
}

TOMA_API int toma_merge_recompute(const toma_desc *desc, const void *X, const int32_t *idx, float *Z, void *wcache,
                                  void *Xm, void *ws, size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!X || !idx || !Z || !wcache || !Xm) return TOMA_ERR_NULL;
  if (misaligned(X, 16) || misaligned(Xm, 16) || misaligned(Z, 4) || misaligned(idx, 4) || misaligned(wcache, 256))
    return TOMA_ERR_ALIGN;
  return launch_merge_fused(s, X, idx, Z, Xm, static_cast<char *>(wcache), w, static_cast<hipStream_t>(stream));
}

TOMA_API int toma_unmerge_recompute(const toma_desc *desc, const void *X, const int32_t *idx, const float *Z,
                                    const void *wcache, const void *O, int32_t o_rows, void *Y, void *ws,
                                    size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!X || !idx || !Z || !wcache || !O || !Y) return TOMA_ERR_NULL;
  if (o_rows < s.D) return TOMA_ERR_SHAPE;
  if (misaligned(X, 16) || misaligned(O, 16) || misaligned(Y, 16) || misaligned(Z, 4) || misaligned(idx, 4) ||
      misaligned(wcache, 256))
    return TOMA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char *wsb = static_cast<char *>(ws);
  rc = launch_scale_rows(s, O, Z, o_rows, wsb + w.os, st);
  if (rc != TOMA_OK) return rc;
  return launch_unmerge_fused(s, X, idx, static_cast<const char *>(wcache), wsb + w.os, s.D, Y, w, st);
}

TOMA_API int toma_unmerge_pinv(const toma_desc *desc, const void *A, const float *Z, const void *O, int32_t o_rows,
                               float rcond, void *Y, void *ws, size_t ws_bytes, void *stream) {
  Shape s; Workspace w;
  int rc = prepare(desc, nullptr, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (!A || !Z || !O || !Y) return TOMA_ERR_NULL;
  if (o_rows < s.D || !(rcond >= 0.0f) || !(rcond < 1.0f)) return TOMA_ERR_SHAPE;
  if (misaligned(A, 16) || misaligned(O, 16) || misaligned(Y, 16) || misaligned(Z, 4)) return TOMA_ERR_ALIGN;
  return launch_unmerge_pinv(s, A, Z, O, o_rows, rcond, Y, static_cast<char *>(ws), w,
                             static_cast<hipStream_t>(stream));
}

TOMA_API int toma_layer(const toma_desc *desc, const toma_attn_desc *attn, uint32_t reuse_flags, const void *X,
                        const void *X_extra_opt, int32_t *idx, void *A, float *Z, void *amap, const void *Wq,
                        const void *Wk, const void *Wv, const void *Wo_opt, void *Y, void *Y_extra_opt,
                        void *ws, size_t ws_bytes, void *stream) {
  if (!attn) return TOMA_ERR_NULL;
  Shape s; Workspace w;
  int rc = prepare(desc, attn, ws, ws_bytes, &s, &w);
  if (rc != TOMA_OK) return rc;
  if (reuse_flags & ~(uint32_t)(TOMA_REUSE_IDX | TOMA_REUSE_A | TOMA_RECOMPUTE_WEIGHTS)) return TOMA_ERR_UNSUPPORTED;
  const bool recompute = (reuse_flags & TOMA_RECOMPUTE_WEIGHTS) != 0;
  if (recompute && (reuse_flags & TOMA_REUSE_A)) return TOMA_ERR_UNSUPPORTED;  // there is no A to reuse
  const bool reuse_a = (reuse_flags & TOMA_REUSE_A) != 0;
  const bool reuse_idx = reuse_a || (reuse_flags & TOMA_REUSE_IDX) != 0;
  if (!X || (!A && !recompute) || !Z || !Wq || !Wk || !Wv || !Y) return TOMA_ERR_NULL;
  if (!reuse_a && !idx) return TOMA_ERR_NULL;
  if ((s.T > 0) != (X_extra_opt != nullptr) || (s.T > 0) != (Y_extra_opt != nullptr)) return TOMA_ERR_NULL;
  if (misaligned(X, 16) || misaligned(A, 16) || misaligned(Y, 16) || misaligned(Z, 4) || misaligned(Wq, 16) ||
      misaligned(Wk, 16) || misaligned(Wv, 16) || (idx && misaligned(idx, 4)) ||
      (X_extra_opt && misaligned(X_extra_opt, 16)) || (Y_extra_opt && misaligned(Y_extra_opt, 16)) ||
      (Wo_opt && misaligned(Wo_opt, 16)))
    return TOMA_ERR_ALIGN;
  rc = recompute ? TOMA_OK : check_map(w, amap);
  if (rc != TOMA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char *wsb = static_cast<char *>(ws);
  uint8_t *occ = static_cast<uint8_t *>(amap);
  // Xm and O are internal to the layer and live in their own workspace sections.
  void *Xm = wsb + w.xm, *O = wsb + w.o;
  if (!reuse_idx) {
    rc = launch_select(s, X, idx, nullptr, nullptr, wsb, w, st);
    if (rc != TOMA_OK) return rc;
  }
  if (recompute) {  // no A: the weights are recomputed inside the merge and again inside the unmerge
    rc = launch_merge_fused(s, X, idx, Z, Xm, wsb + w.fcache, w, st);
  } else {
    if (!reuse_a) {  // (a cached A comes with its map)
      rc = launch_weights(s, X, idx, A, Z, occ, wsb, w, st);
      if (rc != TOMA_OK) return rc;
    }
    rc = launch_merge(s, X, A, Z, !reuse_a, occ, Xm, wsb, w, st);
  }
  if (rc != TOMA_OK) return rc;
  // inside the layer the attention writes its merged rows already divided by Z (the unmerge's
  // input), so no separate scaling pass runs; the extra-token rows go straight to the caller's Y_extra
  rc = launch_attend(s, Xm, X_extra_opt, Wq, Wk, Wv, Wo_opt, O, Z, s.T > 0 ? Y_extra_opt : nullptr, wsb, w, st);
  if (rc != TOMA_OK) return rc;
  rc = recompute ? launch_unmerge_fused(s, X, idx, wsb + w.fcache, O, s.L, Y, w, st)
                 : launch_unmerge(s, A, Z, occ, O, s.L, true, Y, wsb, w, st);
  return rc;
}

TOMA_API int toma_mlp(int32_t dtype, int32_t rows, int32_t C, int32_t hidden, const void *In, const void *W1,
                      const void *W2, void *Hbuf, void *Out, void *stream) {
  if (dtype != TOMA_F32 && dtype != TOMA_BF16) return TOMA_ERR_UNSUPPORTED;
  if (rows <= 0 || C <= 0 || hidden <= 0) return TOMA_ERR_SHAPE;
  if (C % 32 || hidden % 32) return TOMA_ERR_UNSUPPORTED;
  if ((long long)rows * std::max(C, hidden) >= (1ll << 40)) return TOMA_ERR_UNSUPPORTED;
  if (!In || !W1 || !W2 || !Hbuf || !Out) return TOMA_ERR_NULL;
  if (misaligned(In, 16) || misaligned(W1, 16) || misaligned(W2, 16) || misaligned(Hbuf, 16) || misaligned(Out, 16))
    return TOMA_ERR_ALIGN;
  return launch_mlp(dtype, rows, C, hidden, In, W1, W2, Hbuf, Out, static_cast<hipStream_t>(stream));
}
