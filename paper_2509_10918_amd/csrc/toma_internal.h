// Host-side plumbing shared by the C-ABI entry points: validated shapes, workspace layout and
// the launchers each stage file exports.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

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
  size_t sim, stats, lse, zpart, os, q, k, v, oh, xm, o, total;
  int stat_parts, z_parts;
};

constexpr int kGemmMinTile = 64;  // smallest block tile edge of the MFMA GEMM kernels

int make_shape(const toma_desc *d, const toma_attn_desc *a, Shape *s);
void plan_workspace(const Shape &s, Workspace *w);

// stage launchers (each returns a toma_status)
int launch_select(const Shape &s, const void *X, int32_t *idx, float *gain, char *ws, const Workspace &w,
                  hipStream_t st);
int launch_weights(const Shape &s, const void *X, const int32_t *idx, void *A, float *Z, char *ws,
                   const Workspace &w, hipStream_t st);
int launch_merge(const Shape &s, const void *X, const void *A, const float *Z, void *Xm, hipStream_t st);
// Zs (optional): divide the merged rows of O by max(Z, 1e-20) on the way out (the unmerge input)
int launch_attend(const Shape &s, const void *Xm, const void *Xe, const void *Wq, const void *Wk,
                  const void *Wv, const void *Wo, void *O, const float *Zs, char *ws, const Workspace &w,
                  hipStream_t st);
// prescaled: the merged rows of O were already divided by Z (see launch_attend)
int launch_unmerge(const Shape &s, const void *A, const float *Z, const void *O, int o_rows, bool prescaled,
                   void *Y, char *ws, const Workspace &w, hipStream_t st);
int launch_copy_extra(const Shape &s, const void *O, void *Y_extra, hipStream_t st);

// Kernel identifiers of the profiling aid (toma_profile_*): one per kernel of the path.
enum KernelId { K_GRAM = 0, K_GREEDY, K_WSTATS, K_LSE, K_WWRITE, K_ZSUM, K_MERGE, K_QKV, K_ATTN, K_PROJ,
                K_SCALE, K_UNMERGE, K_COPY, K_COUNT };

// Brackets one launch with HIP events on its stream while profiling is enabled; free otherwise.
struct KernelTimer {
  KernelTimer(int id, hipStream_t st);
  ~KernelTimer();
  int slot;
  hipStream_t st;
};

inline int launch_status() { return hipGetLastError() == hipSuccess ? TOMA_OK : TOMA_ERR_LAUNCH; }

}  // namespace toma
