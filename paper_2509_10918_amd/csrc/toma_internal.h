// Host-side plumbing shared by the C-ABI entry points: validated shapes, workspace layout and
// the launchers each stage file exports.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <algorithm>

#include "../../include/toma.h"

namespace toma {

struct Shape {
  int B, H, W, C, tile_h, tile_w, d_loc, R;
  int N, P, n_loc, D, Nr, Dr;  // Nr, Dr: sources / destinations per merge region
  float scale;                 // logit multiplier of the merge weights
  int dtype;
  int heads, head_dim, T, L;   // attention (0 when no toma_attn_desc was given)
};

// Offsets (bytes) of the scratch sections inside the caller's workspace.
struct Workspace {
  size_t sim, gram, stats, lse, zpart, os, q, k, v, oh, xm, o, split, pinv, fcache, total;
  int stat_parts, z_parts;
  // occupancy map of A, kept by the caller next to (A, Z): blocks of kOccDest destinations x kOccSrc
  // sources per merge region (0: this shape uses none)
  int occ_db, occ_sb;
  size_t occ_bytes;
  // fresh weights: Z comes out of the merge product (row sums of its own A fragments) instead of a
  // reduction of the weights kernel's partial sums; needs K whole in every workgroup of that product
  bool z_in_merge;
};

// Occupancy map of the stored merge weights.  With a small temperature almost every source token
// puts all of its weight on one or two destinations and the rest of its column of A rounds to an
// exact zero: the merge and unmerge products then multiply blocks of zeros.  A byte per
// (kOccDest destinations x kOccSrc sources) block of A says whether the block holds any nonzero
// value; the two products skip the K steps whose blocks are all empty, which changes no result
// (finite inputs) and costs one read of A.  Worth it when the products are long enough.
constexpr int kOccDest = 128, kOccSrc = 32;
inline bool occupancy_pays(int Nr, int Dr, int C, int elem_size) {
  // long products only (the map costs a kernel of its own unless the single-pass weights kernel
  // writes it); a K list holds at most 1024 steps
  return Nr >= 2048 && Dr >= 1024 && Nr % kOccSrc == 0 && Dr % kOccDest == 0 && (C * elem_size) % 128 == 0 &&
         Nr / (128 / elem_size) <= 1024 && Dr / (128 / elem_size) <= 1024;
}

constexpr int kGemmMinSlice = 16;  // narrowest wave slice of a GEMM block tile (rows or columns)

// ---- shape planning of the load-to-LDS GEMM (host side; the workspace layout depends on it) ----
// The kernel needs K to be a multiple of its K step (128 bytes of elements) and at least one
// 16-byte packet of rows and columns.
inline bool gemm_async_fits(int M, int N, int K, int elem_size) {
  const int bk = 128 / elem_size, epp = 16 / elem_size;
  return K % bk == 0 && M >= epp && N >= epp;
}
struct GemmPlan { int bm, bn, nsplit; double cost; };  // cost: estimated shader clocks
// Cost model in shader clocks, fitted to measurements of the kernel on MI355X (sweeps of every tile
// and split on the SDXL-sized products): a K step of a workgroup costs about step[][] (it depends on
// which operands are k-major: their fragment reads go through the LDS transpose path), a workgroup
// pays a fixed prologue + epilogue (epi weighs the epilogue: 1 = plain stores, 3 = the softmax
// statistics / exponentials of the merge weights), and the grid runs in rounds of one workgroup per
// CU (two for the narrow tiles).  Splitting K adds a pass that reads every fp32 partial tile and
// writes the output.
inline GemmPlan plan_gemm_async(int M, int N, int K, int batch, int elem_size, bool may_split, bool a_ks, bool b_ks,
                                int epi) {
  static const int bm[5] = {256, 256, 128, 128, 64}, bn[5] = {256, 128, 128, 64, 64};
  static const int step[3][5] = {{3230, 2200, 1230, 1000, 560},   // both operands k-contiguous
                                 {3700, 1900, 1300, 810, 560},    // one k-major
                                 {3400, 2100, 1220, 750, 560}};   // both k-major
  static const int per_cu[5] = {1, 1, 1, 2, 2};
  const int kind = (a_ks ? 1 : 0) + (b_ks ? 1 : 0);
  const int nk = K / (128 / elem_size);
  GemmPlan best{128, 128, 1, 0.0};
  double best_cost = -1.0;
  for (int i = 0; i < 5; i++) {
    const long long tiles = (long long)((M + bm[i] - 1) / bm[i]) * ((N + bn[i] - 1) / bn[i]) * batch;
    for (int ns = 1; ns <= (may_split ? 8 : 1); ns++) {
      if (ns > 1 && nk / ns < 8) break;
      const long long blocks = tiles * ns, slots = 256ll * per_cu[i];
      const long long rounds = (blocks + slots - 1) / slots;
      const double fixed = 4000.0 + epi * bm[i] * bn[i] / 8.0;
      const long long share = std::min<long long>(per_cu[i], (blocks + 255) / 256);  // workgroups sharing a CU
      double cost = rounds * (((nk + ns - 1) / ns) * (double)step[kind][i] * share + fixed);
      if (ns > 1) cost += 8000.0 + (4.0 * ns + elem_size) * (double)M * N * batch / 1500.0;
      if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = GemmPlan{bm[i], bn[i], ns, cost}; }
    }
  }
  return best;
}

// Tile and K split of the merge (M = destinations, K = sources) and unmerge (M = sources, K =
// destinations) products of a merge region.  With a block map the work per workgroup is not known on
// the host: splitting K would mostly split empty steps, so K stays whole unless the tiles alone
// cannot occupy the chip.
inline GemmPlan plan_map_product(int M, int N, int K, int batch, int elem_size, bool a_ks, bool b_ks, bool has_map) {
  bool may_split = true;
  if (has_map && (long long)((M + 127) / 128) * ((N + 127) / 128) * batch >= 128) may_split = false;
  return plan_gemm_async(M, N, K, batch, elem_size, may_split, a_ks, b_ks, 1);
}

// The single-pass merge-weight kernel keeps a (32 sources) x (all destinations of the merge region)
// logit tile in the accumulators of one workgroup: it needs the destinations of a region to be
// 128 * {1, 2, 4, 8, 16}, the sources a multiple of 32, and rows of a multiple of 128 bytes.
inline bool weights_fused_fits(int Nr, int Dr, int C, int elem_size) {
  const int nj = Dr / 128;
  return Dr % 128 == 0 && (nj == 1 || nj == 2 || nj == 4 || nj == 8 || nj == 16) && Nr % 32 == 0 &&
         (C * elem_size) % 128 == 0;
}

// Single pass or two passes for the merge weights?  The single-pass kernel streams every destination
// row through each of its workgroups: about 4 clocks per destination row and K step (measured: it is
// bound by what one CU can pull in), in rounds of one workgroup per CU, plus a fixed part.  The two
// passes cost two planned products plus the small kernel between them.  Few, long rows (a Flux
// block: 1024 destinations, 48 K steps, 128 workgroups) favour the two passes; many destinations
// with a short K favour the single pass.
inline bool weights_single_pass(int Nr, int Dr, int C, int batch, int elem_size) {
  if (!weights_fused_fits(Nr, Dr, C, elem_size)) return false;
  if (!gemm_async_fits(Nr, Dr, C, elem_size)) return true;
  const long long wgs = (long long)(Nr / 32) * batch;
  const double rounds = (double)((wgs + 255) / 256);
  const double single = 19000.0 + rounds * (C * elem_size / 128) * Dr * 4.0;
  const double two = 2.0 * plan_gemm_async(Nr, Dr, C, batch, elem_size, false, false, false, 3).cost + 14000.0;
  return single <= two;
}

int make_shape(const toma_desc *d, const toma_attn_desc *a, Shape *s);
void plan_workspace(const Shape &s, Workspace *w);

// stage launchers (each returns a toma_status)
// Similarities of bf16 tokens on the int8 matrix cores (toma_gram_i8.hip): scratch size (0: this shape
// takes the fp64 kernel instead) and launch; nrm_out / flag_out: per-token norms and the flags of tokens
// whose rows of S the selection kernel has to recompute in double precision
size_t gram_i8_workspace_bytes(const Shape &s);
int launch_gram_i8(const Shape &s, const void *X, int32_t *S, char *ws_part, const double **nrm_out,
                   const uint8_t **flag_out, hipStream_t st);
// gain, gap: optional outputs (null: not wanted); parts: null, or where the profiling variant of the
// greedy kernel leaves the clocks of the parts of its rounds (eight words per region and wave)
int launch_select(const Shape &s, const void *X, int32_t *idx, float *gain, float *gap, char *ws,
                  const Workspace &w, hipStream_t st, unsigned long long *parts = nullptr);
// Pass 1 of the merge weights alone: stats[region][source][part] = (largest logit, sum of exponentials)
// over each slice of *slice destinations, lse[region][source] = log-sum-exp over all destinations,
// lse2 = the same as (largest logit, log of the sum)
int launch_weight_stats(const Shape &s, const void *X, const int32_t *idx, float2 *stats, int stat_parts, float *lse,
                        float2 *lse2, int *slice, hipStream_t st);
// occ: the occupancy map that travels with (A, Z), w.occ_bytes bytes (null iff the shape uses none).
// launch_weights writes it along with A and Z; launch_occupancy rebuilds it from a stored A;
// launch_merge / launch_unmerge read it.
int launch_weights(const Shape &s, const void *X, const int32_t *idx, void *A, float *Z, uint8_t *occ, char *ws,
                   const Workspace &w, hipStream_t st);
int launch_occupancy(const Shape &s, const void *A, uint8_t *occ, const Workspace &w, hipStream_t st);
// make_z: the weights are fresh and launch_weights left Z to this product (w.z_in_merge): Z is written;
// otherwise Z is read
int launch_merge(const Shape &s, const void *X, const void *A, float *Z, bool make_z, const uint8_t *occ, void *Xm,
                 char *ws, const Workspace &w, hipStream_t st);
// Zs (optional): divide the merged rows of O by max(Z, 1e-20) on the way out (the unmerge input)
// O_extra (optional): the extra-token rows go to O_extra [B, T, C] instead of rows D.. of O
int launch_attend(const Shape &s, const void *Xm, const void *Xe, const void *Wq, const void *Wk,
                  const void *Wv, const void *Wo, void *O, const float *Zs, void *O_extra, char *ws,
                  const Workspace &w, hipStream_t st);
// U: [B, L, C] query tokens; Ctx: [B, t_ctx, c_ctx] context tokens; Wk, Wv: [c_ctx, C]
int launch_cross_attend(const Shape &s, const void *U, const void *Ctx, int t_ctx, int c_ctx, const void *Wq,
                        const void *Wk, const void *Wv, const void *Wo, void *O, char *ws, const Workspace &w,
                        hipStream_t st);
// prescaled: the merged rows of O were already divided by Z (see launch_attend)
int launch_unmerge(const Shape &s, const void *A, const float *Z, const uint8_t *occ, const void *O, int o_rows,
                   bool prescaled, void *Y, char *ws, const Workspace &w, hipStream_t st);
// Os[b][j] = O[b][j] / max(Z[b][j], 1e-20) for the D merged rows of every sample
int launch_scale_rows(const Shape &s, const void *O, const float *Z, int o_rows, void *Os, hipStream_t st);
// Merge / unmerge with the weights recomputed instead of read from a stored A.  cache: fused_cache_bytes()
// bytes written by launch_merge_fused (log-sum-exp per source and the statistics that say which tiles of
// weights are empty) and read by launch_unmerge_fused; Os as for launch_unmerge with prescaled rows.
size_t fused_cache_bytes(const Shape &s, const Workspace &w);
int launch_merge_fused(const Shape &s, const void *X, const int32_t *idx, float *Z, void *Xm, char *cache,
                       const Workspace &w, hipStream_t st);
int launch_unmerge_fused(const Shape &s, const void *X, const int32_t *idx, const char *cache, const void *Os,
                         int os_rows, void *Y, const Workspace &w, hipStream_t st);
// Y = (A / Z)^+ O with singular values <= rcond * largest dropped; merge regions of up to 128 destinations
size_t pinv_workspace_bytes(const Shape &s);
int launch_unmerge_pinv(const Shape &s, const void *A, const float *Z, const void *O, int o_rows, float rcond, void *Y,
                        char *ws, const Workspace &w, hipStream_t st);
// Out = gelu(In W1) W2 on `rows` rows; Hbuf is [rows, hidden] scratch of the same dtype
int launch_mlp(int dtype, int rows, int C, int hidden, const void *In, const void *W1, const void *W2, void *Hbuf,
               void *Out, hipStream_t st);

// Kernel identifiers of the profiling aid (toma_profile_*): one per kernel of the path.
enum KernelId { K_LIMBS = 0, K_GRAM, K_GREEDY, K_WSTATS, K_LSE, K_WWRITE, K_ZSUM, K_MERGE, K_QKV, K_ATTN, K_PROJ,
                K_SCALE, K_UNMERGE, K_SPLIT, K_MLP_UP, K_MLP_DOWN, K_OCC, K_PINV_EIG, K_PINV_APPLY, K_MERGE_FUSED, K_UNMERGE_FUSED, K_COUNT };

// Brackets one launch with HIP events on its stream while profiling is enabled; free otherwise.
struct KernelTimer {
  KernelTimer(int id, hipStream_t st);
  ~KernelTimer();
  KernelTimer(const KernelTimer &) = delete;
  KernelTimer &operator=(const KernelTimer &) = delete;
  int id;           // -1: profiling was off at construction
  hipEvent_t a, b;
  hipStream_t st;
};

inline int launch_status() { return hipGetLastError() == hipSuccess ? TOMA_OK : TOMA_ERR_LAUNCH; }

}  // namespace toma
