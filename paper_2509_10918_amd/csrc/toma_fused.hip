// Merge and unmerge with the weights recomputed on the fly instead of read from a stored A
// (paper Sec. 4.2.1: the merge weights are scaled dot-product attention, A = SDPA(X, D, I, tau), so
// both Xm = A~ X and Y = A~^T X' are attention-shaped products that never need A in memory).
//
// With lse_s = log sum_j exp(scale <x_idx[j], x_s>) known per source token s (one statistics pass over
// the logits, the same as pass 1 of the stored-weights path), every weight is
//     p_js = exp(scale <x_idx[j], x_s> - lse_s)  <= 1,
// so neither product needs a running maximum or a rescale:
//     merge    Z_j = sum_s p_js,  Xm_j = (sum_s p_js x_s) / Z_j      queries = destinations, keys = values = sources
//     unmerge  Y_s = sum_j p_js (O_j / Z_j)                           queries = sources, keys = destinations
// One kernel serves both (FusedPol says who is query, key and value).  A workgroup of 8 waves owns
// 16 RT queries and all C output channels; per tile of 32 keys it
//   1. computes the 16 RT x 32 logits on the matrix cores, operands straight from memory (the 2 RT
//      16 x 16 tiles go to the 8 waves, which split the channels between them when there are fewer
//      tiles than waves), partial sums to LDS;
//   2. turns them into weights in the element type, row-major in LDS (and adds up Z for the merge);
//   3. multiplies them with the 32 value rows, staged through LDS in chunks of 128 CTC channels and
//      read back transposed: wave w owns CTC 16-channel tiles of every chunk, all queries.
// Key tiles whose weights are all below e^-110 (zero in bf16 and fp32 alike) are skipped: the
// statistics pass left, per source and slice of destinations, the largest logit of the slice; wave 0
// compacts the tiles that may hold a weight into a list first.  With a small temperature that is a
// few percent of them, which is what makes recomputing competitive with reading a stored A.
#include <type_traits>

#include "toma_gemm.h"
#include "toma_internal.h"
#include "toma_region.h"

namespace toma {

constexpr int kFusedKeys = 32;        // keys per tile (one k-step of the second product)
constexpr int kFusedMaxTiles = 2048;  // key tiles per merge region (list capacity)
constexpr float kFusedEmptyGap = 110.0f;

template <typename T, bool UNMERGE> struct FusedPol {
  RegionView<T> v;
  const int32_t *idx;   // [B][D]
  const T *Os;          // unmerge: [B][os_rows][C], rows [0, D) already divided by Z
  int os_rows;
  const float2 *lse;    // [B*R][Nr]: (largest logit, log of the sum of exponentials) of each source's softmax
  const float2 *stats;  // [B*R][Nr][parts]: (largest logit, .) per slice of `slice` destinations
  int parts, slice;
  float scale;
  T *out;               // merge: Xm [B][D][C]; unmerge: Y [B][N][C]
  float *Z;             // merge: out [B][D]
  __device__ __forceinline__ int nq() const { return UNMERGE ? v.Nr : v.Dr; }
  __device__ __forceinline__ int nk() const { return UNMERGE ? v.Dr : v.Nr; }
  __device__ __forceinline__ int dest_token(int b, int rho, int j) const {
    int t = idx[(size_t)b * v.D + rho * v.Dr + j];
    return t < 0 ? 0 : (t >= v.N ? v.N - 1 : t);
  }
  __device__ __forceinline__ const T *q_row(int b, int rho, int m) const {
    return v.X + ((size_t)b * v.N + (UNMERGE ? v.token(rho, m) : dest_token(b, rho, m))) * v.C;
  }
  __device__ __forceinline__ const T *k_row(int b, int rho, int n) const {
    return v.X + ((size_t)b * v.N + (UNMERGE ? dest_token(b, rho, n) : v.token(rho, n))) * v.C;
  }
  __device__ __forceinline__ const T *v_row(int b, int rho, int n) const {
    return UNMERGE ? Os + ((size_t)b * os_rows + rho * v.Dr + n) * v.C : k_row(b, rho, n);
  }
  // may any weight between queries [m0, m1) and keys [n0, n1) be nonzero?
  __device__ __forceinline__ bool tile_active(int z, int m0, int m1, int n0, int n1) const {
    const int s0 = UNMERGE ? m0 : n0, s1 = UNMERGE ? m1 : n1;  // sources
    const int j0 = UNMERGE ? n0 : m0, j1 = UNMERGE ? n1 : m1;  // destinations
    const int p0 = j0 / slice, p1 = min((j1 - 1) / slice, parts - 1);
    for (int s = s0; s < s1; s++) {
      const float2 ml = lse[(size_t)z * v.Nr + s];
      const float l = ml.x + ml.y;
      const float2 *row = stats + ((size_t)z * v.Nr + s) * parts;
      for (int q = p0; q <= p1; q++)
        if (!(row[q].x - l < -kFusedEmptyGap)) return true;
    }
    return false;
  }
};

template <typename T> __device__ __forceinline__ void frag_load_global(Frag<T> &f, const T *p) {
  if constexpr (sizeof(T) == 2) {
    Pkt pk = pkt_load(p);
    f = __builtin_bit_cast(Frag<T>, pk);
  } else {
    struct { Pkt a, b; } two = {pkt_load(p), pkt_load(p + 4)};
    f = __builtin_bit_cast(Frag<T>, two);
  }
}

template <typename T, bool UNMERGE, int RT, int CTC, int NCH>
__global__ __launch_bounds__(512) void k_fused(const FusedPol<T, UNMERGE> pol) {
  constexpr int ES = (int)sizeof(T), EPP = 16 / ES;
  constexpr int BQ = 16 * RT;               // queries per workgroup
  constexpr int NT = 2 * RT;                // 16 x 16 logit tiles per key tile
  constexpr int NSPLIT = 8 / NT;            // waves sharing one logit tile, each a slice of the channels
  constexpr int CW = 128 * CTC;             // channels per chunk of the value tile
  constexpr int LDV = CW + EPP;             // padded row of the value tile
  constexpr int LDP = kFusedKeys + EPP;     // padded row of the weight tile
  constexpr int NPK = kFusedKeys * (CW / EPP) / 512;  // value packets per thread and chunk
  __shared__ __align__(16) T Vt[2][kFusedKeys * LDV];
  __shared__ __align__(16) float Sp[8][256];          // partial logit tiles, [wave][4 r][64 lanes]
  __shared__ __align__(16) T Pt[BQ * LDP];
  __shared__ uint16_t klist[kFusedMaxTiles];
  __shared__ int klist_n;

  const RegionView<T> &v = pol.v;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const int z = blockIdx.y, b = z / v.R, rho = z % v.R;
  const int m0 = blockIdx.x * BQ, NQ = pol.nq(), NK = pol.nk(), C = v.C;
  const int m1 = min(m0 + BQ, NQ);
  const int ntiles = (NK + kFusedKeys - 1) / kFusedKeys;

  // ---- key tiles that may hold a weight for these queries ----
  if (w == 0) {
    int count = 0;
    for (int t0 = 0; t0 < ntiles; t0 += 64) {
      const int kt = t0 + lane;
      const bool act = kt < ntiles && pol.tile_active(z, m0, m1, kt * kFusedKeys, min((kt + 1) * kFusedKeys, NK));
      const uint64_t mask = __ballot(act);
      if (act) klist[count + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)kt;
      count += __popcll(mask);
    }
    if (lane == 0) klist_n = count;
  }
  __syncthreads();
  const int nlist = klist_n;

  // this wave's part of the logits: tile (rt, ct) of the 16 RT x 32 block, channel steps [ks0, ks1)
  const int tile = w % NT, rt = tile >> 1, ct = tile & 1, sp = w / NT;
  const int ksteps = C / 32, ks0 = ksteps * sp / NSPLIT, ks1 = ksteps * (sp + 1) / NSPLIT;
  const T *q_ptr = pol.q_row(b, rho, min(m0 + 16 * rt + c, NQ - 1)) + 8 * g;
  // the weights this thread makes: BQ x 32 values, 4 consecutive keys of one query per item
  constexpr int ITEMS = BQ * kFusedKeys / 4;   // <= 512
  const bool maker = tid < ITEMS;
  const int pm = tid / 8, pk0 = (tid % 8) * 4;  // query row and first key of the item
  float2 bias_q = make_float2(0.f, 0.f);
  if (UNMERGE && maker && m0 + pm < NQ) bias_q = pol.lse[(size_t)z * v.Nr + m0 + pm];
  float zsum = 0.f;  // merge: row sum of the weights of query pm (thread tid % 8 == 0 holds it)

  f32x4 acc[NCH][RT][CTC];
#pragma unroll
  for (int h = 0; h < NCH; h++)
#pragma unroll
    for (int i = 0; i < RT; i++)
#pragma unroll
      for (int j = 0; j < CTC; j++) acc[h][i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  int vb = 0;  // value-tile buffer that the next chunk goes to
  for (int it = 0; it < nlist; it++) {
    const int n0 = (int)klist[it] * kFusedKeys;
    // ---- 1. logits of this wave's tile over its channel slice ----
    const T *k_ptr = pol.k_row(b, rho, min(n0 + 16 * ct + c, NK - 1)) + 8 * g;
    f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int ks = ks0; ks < ks1; ks += 4) {
      Frag<T> fa[4], fb[4];
#pragma unroll
      for (int u = 0; u < 4; u++)
        if (ks + u < ks1) { frag_load_global(fa[u], q_ptr + 32 * (ks + u)); frag_load_global(fb[u], k_ptr + 32 * (ks + u)); }
#pragma unroll
      for (int u = 0; u < 4; u++)
        if (ks + u < ks1) mma16(sacc, fa[u], fb[u]);  // lane: key column c, query rows 4 g + r
    }
#pragma unroll
    for (int r = 0; r < 4; r++) Sp[w][64 * r + lane] = sacc[r];
    // value rows of the first chunk, on their way while the logits settle
    Pkt vreg[NPK];
    auto fetch_values = [&](int ch) {
#pragma unroll
      for (int u = 0; u < NPK; u++) {
        const int q = tid + 512 * u, row = q / (CW / EPP), col = ch * CW + (q % (CW / EPP)) * EPP;
        vreg[u] = col < C ? pkt_load(pol.v_row(b, rho, min(n0 + row, NK - 1)) + col) : pkt_zero();
      }
    };
    auto stash_values = [&](int buf) {
#pragma unroll
      for (int u = 0; u < NPK; u++) {
        const int q = tid + 512 * u, row = q / (CW / EPP), colp = q % (CW / EPP);
        pkt_store(&Vt[buf][row * LDV + colp * EPP], vreg[u]);
      }
    };
    fetch_values(0);
    stash_values(vb);
    __syncthreads();  // logits and the first value chunk are in LDS

    // ---- 2. weights: p = exp(scale * logit - lse), rounded to the element type ----
    if (maker) {
      const int prt = pm >> 4, pr = pm & 15;           // row tile and row inside it
      const int pct = pk0 >> 4, pc = pk0 & 15;         // key tile and first key inside it
      f32x4 lg = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int q = 0; q < NSPLIT; q++)
        lg += *reinterpret_cast<const f32x4 *>(&Sp[q * NT + 2 * prt + pct][64 * (pr & 3) + 16 * (pr >> 2) + pc]);
      alignas(8) T o[4];
      float rowsum = 0.f;
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int n = n0 + pk0 + u;
        float2 bias = bias_q;
        if (!UNMERGE) bias = n < NK ? pol.lse[(size_t)z * v.Nr + n] : make_float2(0.f, 0.f);
        // (logit - largest logit) is small and nearly exact; only then the log of the sum comes off
        float p = (n < NK && m0 + pm < NQ) ? __expf(__builtin_fmaf(lg[u], pol.scale, -bias.x) - bias.y) : 0.f;
        o[u] = from_f32<T>(p);
        rowsum += to_f32(o[u]);
      }
      if (sizeof(T) == 2) *reinterpret_cast<u32x2 *>(&Pt[pm * LDP + pk0]) = *reinterpret_cast<u32x2 *>(o);
      else *reinterpret_cast<u32x4 *>(&Pt[pm * LDP + pk0]) = *reinterpret_cast<u32x4 *>(o);
      if (!UNMERGE) {  // Z sums the weights as they enter the product: fixed order (eight threads of a row, then tiles in list order)
        rowsum += __shfl_xor(rowsum, 1, 64);
        rowsum += __shfl_xor(rowsum, 2, 64);
        rowsum += __shfl_xor(rowsum, 4, 64);
        zsum += rowsum;
      }
    }
    __syncthreads();  // the weights are in LDS

    // ---- 3. out^T += V^T P^T, chunk by chunk of the value rows ----
    Frag<T> fp[RT];
#pragma unroll
    for (int i = 0; i < RT; i++) frag_load_kc(fp[i], &Pt[(16 * i + c) * LDP + 8 * g]);
#pragma unroll
    for (int h = 0; h < NCH; h++) {
      if (h > 0) {
        // (every wave is past the barrier that followed the previous chunk's stash, hence done with the
        // chunk before that one, whose buffer this one takes)
        fetch_values(h);
        stash_values(vb);
        __syncthreads();
      }
      const T *vt = Vt[vb];
#pragma unroll
      for (int j = 0; j < CTC; j++) {
        const int col = 16 * (w * CTC + j);  // inside the chunk
        if (h * CW + col < C) {
          Frag<T> fv;
          frag_load_ks(fv, vt, LDV, 8 * g, 8 * g + 4, col, lane);
#pragma unroll
          for (int i = 0; i < RT; i++) mma16(acc[h][i][j], fv, fp[i]);  // lane: query c, channels 4 g + r
        }
      }
      vb ^= 1;
    }
  }

  // ---- epilogue: lane holds, of query 16 i + c, the channels h CW + 16 (w CTC + j) + 4 g + r ----
  __shared__ float zrow[BQ];
  if (!UNMERGE) {
    if (maker && (tid & 7) == 0) zrow[pm] = zsum;
    __syncthreads();
    if (maker && (tid & 7) == 0 && m0 + pm < NQ) pol.Z[(size_t)b * v.D + rho * v.Dr + m0 + pm] = zsum;
  }
#pragma unroll
  for (int i = 0; i < RT; i++) {
    const int m = m0 + 16 * i + c;
    if (m >= NQ) continue;
    float sc = 1.0f;
    T *dst;
    if (UNMERGE) {
      dst = pol.out + ((size_t)b * v.N + v.token(rho, m)) * C;
    } else {
      sc = 1.0f / fmaxf(zrow[16 * i + c], 1e-20f);
      dst = pol.out + ((size_t)b * v.D + rho * v.Dr + m) * C;
    }
#pragma unroll
    for (int h = 0; h < NCH; h++)
#pragma unroll
      for (int j = 0; j < CTC; j++) {
        const int col = h * CW + 16 * (w * CTC + j) + 4 * g;
        if (col < C) {
          alignas(16) T o[4];
#pragma unroll
          for (int r = 0; r < 4; r++) o[r] = from_f32<T>(acc[h][i][j][r] * sc);
          if (sizeof(T) == 2) *reinterpret_cast<u32x2 *>(dst + col) = *reinterpret_cast<u32x2 *>(o);
          else *reinterpret_cast<u32x4 *>(dst + col) = *reinterpret_cast<u32x4 *>(o);
        }
      }
  }
}

// Shapes the kernel is built for: (RT, CTC, NCH) by channel width, accumulators <= 96 registers.
template <typename T, bool UNMERGE>
static int launch_fused(const Shape &s, const FusedPol<T, UNMERGE> &pol, int kernel_id, hipStream_t st) {
  const int NQ = UNMERGE ? s.Nr : s.Dr, NK = UNMERGE ? s.Dr : s.Nr;
  if ((NK + kFusedKeys - 1) / kFusedKeys > kFusedMaxTiles) return TOMA_ERR_UNSUPPORTED;
  KernelTimer kt(kernel_id, st);
#define TOMA_FUSED_LAUNCH(RT, CTC, NCH)                                                                            \
  hipLaunchKernelGGL((k_fused<T, UNMERGE, RT, CTC, NCH>), dim3((NQ + 16 * RT - 1) / (16 * RT), s.B * s.R), dim3(512), 0, st, pol)
  // Queries per workgroup: a workgroup walks its key tiles one after the other, so the grid should
  // have a workgroup for every CU before a workgroup gets more queries (16 RT, RT = 4, 2 or 1).
  const long long regions = (long long)s.B * s.R;
  auto rt_for = [&](int rt_max) {
    int rt = rt_max;
    while (rt > 1 && ((NQ + 16 * rt - 1) / (16 * rt)) * regions < 256) rt >>= 1;
    return rt;
  };
#define TOMA_FUSED_BY_RT(CTC)                                      \
  switch (rt_for(4)) {                                             \
    case 4: TOMA_FUSED_LAUNCH(4, CTC, 1); break;                   \
    case 2: TOMA_FUSED_LAUNCH(2, CTC, 1); break;                   \
    default: TOMA_FUSED_LAUNCH(1, CTC, 1); break;                  \
  }
  // (chunks of the value tile: two of them, 32 rows each, have to fit the LDS next to the rest)
  if constexpr (sizeof(T) == 2) {
    if (s.C <= 128) { TOMA_FUSED_BY_RT(1) }
    else if (s.C <= 256) { TOMA_FUSED_BY_RT(2) }
    else if (s.C <= 640) { TOMA_FUSED_BY_RT(5) }
    else if (s.C <= 1280) { if (rt_for(2) == 2) TOMA_FUSED_LAUNCH(2, 5, 2); else TOMA_FUSED_LAUNCH(1, 5, 2); }
    else if (s.C <= 3072) TOMA_FUSED_LAUNCH(1, 4, 6);
    else return TOMA_ERR_UNSUPPORTED;
  } else {
    // fp32: 64 queries per workgroup wherever the accumulators allow, so that a wave adds up a logit
    // over all channels in the order the statistics pass did: logit minus largest logit is then exact
    // for the weights that matter, as in the stored-weights kernels (fp32 logits of several hundred
    // leave no room for two independent roundings inside a 1e-4 tolerance)
    if (s.C <= 128) TOMA_FUSED_LAUNCH(4, 1, 1);
    else if (s.C <= 256) TOMA_FUSED_LAUNCH(4, 2, 1);
    else if (s.C <= 768) TOMA_FUSED_LAUNCH(4, 2, 3);
    else if (s.C <= 1280) TOMA_FUSED_LAUNCH(2, 2, 5);
    else if (s.C <= 3072) TOMA_FUSED_LAUNCH(1, 2, 12);
    else return TOMA_ERR_UNSUPPORTED;
  }
#undef TOMA_FUSED_BY_RT
#undef TOMA_FUSED_LAUNCH
  return launch_status();
}

// cache layout: lse2 [B*N] float2, lse [B*N] float (the statistics pass writes it; unused here), statistics
static size_t fused_lse2_bytes(const Shape &s) { return ((size_t)s.B * s.N * sizeof(float2) + 255) & ~(size_t)255; }
static size_t fused_lse_bytes(const Shape &s) { return ((size_t)s.B * s.N * sizeof(float) + 255) & ~(size_t)255; }
size_t fused_cache_bytes(const Shape &s, const Workspace &w) {
  return fused_lse2_bytes(s) + fused_lse_bytes(s) + (size_t)s.B * s.N * w.stat_parts * sizeof(float2);
}

template <typename T>
static int merge_fused_typed(const Shape &s, const void *X, const int32_t *idx, float *Z, void *Xm, char *cache,
                             const Workspace &w, hipStream_t st) {
  float2 *lse2 = reinterpret_cast<float2 *>(cache);
  float *lse = reinterpret_cast<float *>(cache + fused_lse2_bytes(s));
  float2 *stats = reinterpret_cast<float2 *>(cache + fused_lse2_bytes(s) + fused_lse_bytes(s));
  int slice = 0;
  int rc = launch_weight_stats(s, X, idx, stats, w.stat_parts, lse, lse2, &slice, st);
  if (rc != TOMA_OK) return rc;
  FusedPol<T, false> p{};
  p.v = make_view<T>(s, X);
  p.idx = idx; p.Os = nullptr; p.os_rows = 0; p.lse = lse2; p.stats = stats; p.parts = w.stat_parts; p.slice = slice;
  p.scale = s.scale; p.out = static_cast<T *>(Xm); p.Z = Z;
  return launch_fused<T, false>(s, p, K_MERGE_FUSED, st);
}

int launch_merge_fused(const Shape &s, const void *X, const int32_t *idx, float *Z, void *Xm, char *cache,
                       const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? merge_fused_typed<bf16_t>(s, X, idx, Z, Xm, cache, w, st)
                              : merge_fused_typed<float>(s, X, idx, Z, Xm, cache, w, st);
}

template <typename T>
static int unmerge_fused_typed(const Shape &s, const void *X, const int32_t *idx, const char *cache, const void *Os,
                               int os_rows, void *Y, const Workspace &w, hipStream_t st) {
  const float2 *lse2 = reinterpret_cast<const float2 *>(cache);
  const float2 *stats = reinterpret_cast<const float2 *>(cache + fused_lse2_bytes(s) + fused_lse_bytes(s));
  // the slice width of the statistics is a function of the shape: the planner that ran the pass says it
  const int slice = weight_stats_slice(s.Nr, s.Dr, s.C, s.B * s.R, (int)sizeof(T));
  FusedPol<T, true> p{};
  p.v = make_view<T>(s, X);
  p.idx = idx; p.Os = static_cast<const T *>(Os); p.os_rows = os_rows; p.lse = lse2; p.stats = stats;
  p.parts = w.stat_parts; p.slice = slice; p.scale = s.scale; p.out = static_cast<T *>(Y); p.Z = nullptr;
  return launch_fused<T, true>(s, p, K_UNMERGE_FUSED, st);
}

int launch_unmerge_fused(const Shape &s, const void *X, const int32_t *idx, const char *cache, const void *Os,
                         int os_rows, void *Y, const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? unmerge_fused_typed<bf16_t>(s, X, idx, cache, Os, os_rows, Y, w, st)
                              : unmerge_fused_typed<float>(s, X, idx, cache, Os, os_rows, Y, w, st);
}

}  // namespace toma
