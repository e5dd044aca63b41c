// Profiling aid: per-kernel HIP-event timing of the library's own launches (see toma.h).
#include <atomic>
#include <mutex>
#include <string.h>
#include <vector>

#include "toma_internal.h"

namespace toma {

static const char *const kNames[K_COUNT] = {"limbs", "gram", "greedy", "weights_stats", "lse", "weights_write",
                                            "zsum", "merge", "qkv", "attention", "proj", "scale_rows",
                                            "unmerge", "split_finish", "mlp_up", "mlp_down", "occupancy",
                                            "pinv_eig", "pinv_apply", "merge_recompute", "unmerge_recompute"};
struct Rec { int id; hipEvent_t a, b; };
static std::mutex g_mu;
static std::atomic<bool> g_on{false};
static std::vector<Rec> g_recs;
static std::vector<hipEvent_t> g_pool;
static int g_launches[K_COUNT];
static double g_ms[K_COUNT];

static hipEvent_t take_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// The timer owns its two events from construction to destruction and hands the finished pair over
// only then: a toma_profile_read / toma_profile_enable from another thread in between finds either
// nothing of this launch or all of it.
KernelTimer::KernelTimer(int id_, hipStream_t s) : id(-1), a(nullptr), b(nullptr), st(s) {
  if (!g_on.load(std::memory_order_relaxed)) return;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    a = take_event();
    b = take_event();
    if (!a || !b) {
      if (a) g_pool.push_back(a);
      if (b) g_pool.push_back(b);
      a = b = nullptr;
      return;
    }
  }
  id = id_;
  (void)hipEventRecord(a, st);
}

KernelTimer::~KernelTimer() {
  if (id < 0) return;
  (void)hipEventRecord(b, st);
  std::lock_guard<std::mutex> lk(g_mu);
  g_recs.push_back(Rec{id, a, b});
}

static void collect() {
  for (const Rec &r : g_recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      g_launches[r.id]++;
      g_ms[r.id] += ms;
    }
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
}

}  // namespace toma

using namespace toma;
#define TOMA_API extern "C" __attribute__((visibility("default")))

TOMA_API int toma_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  collect();
  g_on.store(on != 0);
  for (int i = 0; i < K_COUNT; i++) { g_launches[i] = 0; g_ms[i] = 0.0; }
  return TOMA_OK;
}

TOMA_API const char *toma_profile_kernel_name(int i) { return (i >= 0 && i < K_COUNT) ? kNames[i] : nullptr; }

TOMA_API int toma_profile_read(const char *kernel, int32_t *launches, float *total_ms) {
  if (!kernel || !launches || !total_ms) return TOMA_ERR_NULL;
  std::lock_guard<std::mutex> lk(g_mu);
  collect();
  for (int i = 0; i < K_COUNT; i++)
    if (strcmp(kernel, kNames[i]) == 0) {
      *launches = g_launches[i];
      *total_ms = (float)g_ms[i];
      g_launches[i] = 0;
      g_ms[i] = 0.0;
      return TOMA_OK;
    }
  return TOMA_ERR_UNSUPPORTED;
}

TOMA_API int toma_profile_map_product(const toma_desc *desc, int which, int32_t *out3) {
  if (!out3) return TOMA_ERR_NULL;
  Shape s;
  int rc = make_shape(desc, nullptr, &s);
  if (rc != TOMA_OK) return rc;
  Workspace w;
  plan_workspace(s, &w);
  const int es = s.dtype == TOMA_BF16 ? 2 : 4;
  if (which == 2) {  // the write pass of the two-pass weights: sources x destinations
    if (weights_single_pass(s.Nr, s.Dr, s.C, s.B * s.R, es) || !gemm_async_fits(s.Nr, s.Dr, s.C, es)) return TOMA_ERR_UNSUPPORTED;
    const GemmPlan pl = plan_gemm_async(s.Nr, s.Dr, s.C, s.B * s.R, es, false, false, false, 3);
    out3[0] = pl.bm; out3[1] = pl.bn; out3[2] = pl.nsplit;
    return TOMA_OK;
  }
  const int M = which == 0 ? s.Dr : s.Nr, K = which == 0 ? s.Nr : s.Dr;
  if ((which != 0 && which != 1) || !gemm_async_fits(M, s.C, K, es)) return TOMA_ERR_UNSUPPORTED;
  const GemmPlan pl = plan_map_product(M, s.C, K, s.B * s.R, es, which == 1, true, w.occ_sb != 0);
  out3[0] = pl.bm; out3[1] = pl.bn; out3[2] = pl.nsplit;
  return TOMA_OK;
}

TOMA_API int toma_profile_greedy_parts(const toma_desc *desc, const void *X, int32_t *idx, uint64_t *parts, void *ws,
                                       size_t ws_bytes, void *stream) {
  Shape s;
  int rc = make_shape(desc, nullptr, &s);
  if (rc != TOMA_OK) return rc;
  Workspace w;
  plan_workspace(s, &w);
  if (!X || !idx || !parts || !ws) return TOMA_ERR_NULL;
  if (ws_bytes < w.total) return TOMA_ERR_WORKSPACE;
  if (((uintptr_t)X & 15) || ((uintptr_t)ws & 255) || ((uintptr_t)parts & 7) || ((uintptr_t)idx & 3)) return TOMA_ERR_ALIGN;
  if (s.n_loc != 256 && s.n_loc != 64) return TOMA_ERR_UNSUPPORTED;
  static_assert(sizeof(unsigned long long) == sizeof(uint64_t), "clock words");
  return launch_select(s, X, idx, nullptr, nullptr, static_cast<char *>(ws), w, static_cast<hipStream_t>(stream),
                       reinterpret_cast<unsigned long long *>(parts));
}
