// Destination selection: cosine similarity inside each region and the greedy facility-location
// pick sequence (paper Sec. 4.1, Eq. 2, Alg. 2; regions as in Alg. 3 step 1).
//
// Three kernels:
//   k_norms   ||x_n||_2 of every token, accumulated in double.
//   k_gram    S = cos(x_i, x_j) per region with the fp64 matrix cores (v_mfma_f64_16x16x4_f64):
//             products of stored bf16 / fp32 values are exact in double, so S is the similarity
//             to ~1e-16 before it is rounded once to the nearest multiple of 2^-25 and stored as
//             a 32-bit integer.  From there on every sum and comparison of the greedy loop is
//             exact integer arithmetic: the picks do not depend on any summation order, and
//             mathematically tied candidates (common: two tokens that only improve each other's
//             coverage) are exact ties that go to the lowest index.
//   k_greedy  one workgroup per (sample, region).  The region's whole S (up to 256 x 256 words)
//             lives in the workgroup's vector registers: wave w owns rows 16w .. 16w+15, lane
//             (g, c) = (lane / 16, lane % 16) holds rows 16w + 4g + r and columns c + 16t.  A
//             round is: per-lane partial sums of max(0, S_ij - m_j), a 16-lane reduction, an
//             in-wave argmax, one LDS exchange between the waves (each wave also posts its
//             candidate's row, so the winner's row is already there for m <- max(m, S_t)).
#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

// Similarities are decided on a grid of 2^-25: |S| <= 1 + rounding, so a lane's 16-term partial
// sum of differences stays below 2^31 and a full 256-term sum below 2^35 (exact in a double).
constexpr double kSimScale = 33554432.0;

// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_norms(const T *__restrict__ X, double *__restrict__ nrm, int rows, int C) {
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T *x = X + (size_t)row * C;
  double acc = 0.0;
  for (int c = lane; c < C; c += kWave) {
    double v = (double)to_f32(x[c]);
    acc += v * v;
  }
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) acc += wave_xor_f64(acc, m);
  if (lane == 0) {
    double n = sqrt(acc);
    nrm[row] = n > 1e-12 ? n : 1e-12;
  }
}

// ------------------------------------------------------------------------------------------------
// 64 x 64 block of one region's similarity matrix per workgroup, 2 x 2 waves of 32 x 32.
template <typename T>
__global__ __launch_bounds__(256) void k_gram(const T *__restrict__ X, const double *__restrict__ nrm,
                                             int32_t *__restrict__ S, RegionMap map, int N, int C, int P,
                                             int n_loc) {
  constexpr int BK = 32;
  constexpr int EPP = 16 / (int)sizeof(T);
  constexpr int LDK = BK + EPP;
  constexpr int PPR = BK / EPP;
  constexpr int NP = 64 * PPR / 256;
  __shared__ __align__(16) T As[64 * LDK];
  __shared__ __align__(16) T Bs[64 * LDK];

  const int bp = blockIdx.z, b = bp / P, p = bp % P;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
  const int g = lane >> 4, c = lane & 15;
  const T *Xb = X + (size_t)b * N * C;

  const T *pa[NP], *pb[NP];
  int lo[NP];
#pragma unroll
  for (int i = 0; i < NP; i++) {
    int q = tid + 256 * i, row = q / PPR, kp = q % PPR;
    lo[i] = row * LDK + kp * EPP;
    int la = m0 + row, lb = n0 + row;
    pa[i] = la < n_loc ? Xb + (size_t)map.token(p, la) * C + kp * EPP : nullptr;
    pb[i] = lb < n_loc ? Xb + (size_t)map.token(p, lb) * C + kp * EPP : nullptr;
  }

  f64x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) acc[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};

  for (int k0 = 0; k0 < C; k0 += BK) {
    Pkt ra[NP], rb[NP];
#pragma unroll
    for (int i = 0; i < NP; i++) {
      ra[i] = pa[i] ? pkt_load(pa[i] + k0) : pkt_zero();
      rb[i] = pb[i] ? pkt_load(pb[i] + k0) : pkt_zero();
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NP; i++) {
      pkt_store(As + lo[i], ra[i]);
      pkt_store(Bs + lo[i], rb[i]);
    }
    __syncthreads();
    Frag<T> fa[2], fb[2];
#pragma unroll
    for (int i = 0; i < 2; i++) {
      frag_load_kc(fa[i], As + (wm * 32 + 16 * i + c) * LDK + 8 * g);
      frag_load_kc(fb[i], Bs + (wn * 32 + 16 * i + c) * LDK + 8 * g);
    }
#pragma unroll
    for (int s = 0; s < 8; s++)
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)to_f32(fa[i].v[s]), (double)to_f32(fb[j].v[s]),
                                                           acc[i][j], 0, 0, 0);
  }

  // fp64 accumulator tile: lane holds column lane % 16 and rows (lane / 16) + 4 r.
  const double *nb = nrm + (size_t)b * N;
  int32_t *Sr = S + (size_t)bp * n_loc * n_loc;
#pragma unroll
  for (int j = 0; j < 2; j++) {
    int col = n0 + wn * 32 + 16 * j + c;
    if (col >= n_loc) continue;
    double ncol = nb[map.token(p, col)];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        int row = m0 + wm * 32 + 16 * i + g + 4 * r;
        if (row < n_loc) {
          double den = nb[map.token(p, row)] * ncol;
          Sr[(size_t)row * n_loc + col] = (int32_t)rint(acc[i][j][r] / den * kSimScale);
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(64 * NT) void k_greedy(const int32_t *__restrict__ S, int32_t *__restrict__ idx,
                                                   float *__restrict__ gain_out, RegionMap map, int P, int d_loc) {
  constexpr int NL = 16 * NT;
  __shared__ int32_t rowbuf[2][NT][NL];
  __shared__ double cand_gain[2][NT];
  __shared__ int cand_idx[2][NT];

  const int bp = blockIdx.x, p = bp % P;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  const int32_t *Sr = S + (size_t)bp * NL * NL;
  const int row0 = 16 * w + 4 * g;

  int32_t s[4][NT];
#pragma unroll
  for (int r = 0; r < 4; r++)
#pragma unroll
    for (int t = 0; t < NT; t++) s[r][t] = Sr[(size_t)(row0 + r) * NL + c + 16 * t];

  int32_t m[NT];
#pragma unroll
  for (int t = 0; t < NT; t++) m[t] = 0;
  unsigned chosen = 0;  // bit r: row row0 + r is already a destination
  const double kNone = -__builtin_inf();

  for (int step = 0; step < d_loc; step++) {
    int32_t part[4] = {0, 0, 0, 0};
    if (step == 0) {
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int r = 0; r < 4; r++) part[r] += s[r][t];
    } else {
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int r = 0; r < 4; r++) part[r] += max(s[r][t] - m[t], 0);
    }
    double acc[4];
#pragma unroll
    for (int r = 0; r < 4; r++) {
      acc[r] = (double)part[r];
#pragma unroll
      for (int x = 1; x < 16; x <<= 1) acc[r] += wave_xor_f64(acc[r], x);
    }
    // best row of this lane group, then of the wave; equal values keep the lower row index
    double bg = kNone;
    int bi = NL;
#pragma unroll
    for (int r = 0; r < 4; r++) {
      bool free_row = !((chosen >> r) & 1u);
      if (free_row && acc[r] > bg) { bg = acc[r]; bi = row0 + r; }
    }
#pragma unroll
    for (int x = 16; x < 64; x <<= 1) {
      double og = wave_xor_f64(bg, x);
      int oi = __shfl_xor(bi, x, 64);
      if (og > bg || (og == bg && oi < bi)) { bg = og; bi = oi; }
    }
    const int buf = step & 1;
    if (bi < NL && g == ((bi & 15) >> 2)) {
      const int rr = bi & 3;
#pragma unroll
      for (int t = 0; t < NT; t++) {
        int32_t v = rr == 0 ? s[0][t] : rr == 1 ? s[1][t] : rr == 2 ? s[2][t] : s[3][t];
        rowbuf[buf][w][c + 16 * t] = v;
      }
    }
    if (lane == 0) { cand_gain[buf][w] = bg; cand_idx[buf][w] = bi; }
    __syncthreads();
    double G = kNone;
    int I = NL, ww = 0;
#pragma unroll
    for (int v = 0; v < NT; v++) {
      double og = cand_gain[buf][v];
      int oi = cand_idx[buf][v];
      if (og > G || (og == G && oi < I)) { G = og; I = oi; ww = v; }
    }
#pragma unroll
    for (int t = 0; t < NT; t++) {
      int32_t mv = rowbuf[buf][ww][c + 16 * t];
      m[t] = step == 0 ? mv : max(m[t], mv);
    }
    if (w == (I >> 4) && g == ((I & 15) >> 2)) chosen |= 1u << (I & 3);
    if (threadIdx.x == 0) {
      idx[(size_t)bp * d_loc + step] = map.token(p, I);
      if (gain_out) gain_out[(size_t)bp * d_loc + step] = (float)(G / kSimScale);
    }
  }
}

template <typename T>
static int select_typed(const Shape &s, const T *X, int32_t *idx, float *gain, char *ws, const Workspace &w,
                        hipStream_t st) {
  double *nrm = reinterpret_cast<double *>(ws + w.nrm);
  int32_t *S = reinterpret_cast<int32_t *>(ws + w.sim);
  RegionMap map{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  int rows = s.B * s.N;
  { KernelTimer kt(K_NORMS, st);
  hipLaunchKernelGGL(k_norms<T>, dim3((rows + 3) / 4), dim3(256), 0, st, X, nrm, rows, s.C); }
  int tiles = (s.n_loc + 63) / 64;
  { KernelTimer kt(K_GRAM, st);
  hipLaunchKernelGGL(k_gram<T>, dim3(tiles, tiles, s.B * s.P), dim3(256), 0, st, X, nrm, S, map, s.N, s.C, s.P,
                     s.n_loc); }
  int regions = s.B * s.P;
  KernelTimer kt(K_GREEDY, st);
  switch (s.n_loc / 16) {
#define TOMA_GREEDY_CASE(NT)                                                                              \
  case NT:                                                                                                \
    hipLaunchKernelGGL(k_greedy<NT>, dim3(regions), dim3(64 * NT), 0, st, S, idx, gain, map, s.P, s.d_loc); \
    break;
    TOMA_GREEDY_CASE(1)
    TOMA_GREEDY_CASE(2)
    TOMA_GREEDY_CASE(3)
    TOMA_GREEDY_CASE(4)
    TOMA_GREEDY_CASE(5)
    TOMA_GREEDY_CASE(6)
    TOMA_GREEDY_CASE(7)
    TOMA_GREEDY_CASE(8)
    TOMA_GREEDY_CASE(9)
    TOMA_GREEDY_CASE(10)
    TOMA_GREEDY_CASE(11)
    TOMA_GREEDY_CASE(12)
    TOMA_GREEDY_CASE(13)
    TOMA_GREEDY_CASE(14)
    TOMA_GREEDY_CASE(15)
    TOMA_GREEDY_CASE(16)
#undef TOMA_GREEDY_CASE
    default:
      return TOMA_ERR_UNSUPPORTED;
  }
  return launch_status();
}

int launch_select(const Shape &s, const void *X, int32_t *idx, float *gain, char *ws, const Workspace &w,
                  hipStream_t st) {
  if (s.dtype == TOMA_BF16) return select_typed<bf16_t>(s, static_cast<const bf16_t *>(X), idx, gain, ws, w, st);
  return select_typed<float>(s, static_cast<const float *>(X), idx, gain, ws, w, st);
}

}  // namespace toma
