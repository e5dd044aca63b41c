// Destination selection: cosine similarity inside each region and the greedy facility-location
// pick sequence (paper Sec. 4.1, Eq. 2, Alg. 2; regions as in Alg. 3 step 1).
//
// Two kernels:
//   k_gram    S = cos(x_i, x_j) per region with the fp64 matrix cores (v_mfma_f64_16x16x4_f64):
//             products of stored bf16 / fp32 values are exact in double, so S is the similarity
//             to ~1e-16 before it is rounded once to the nearest multiple of 2^-22 and stored as
//             a 32-bit integer.  From there on every sum and comparison of the greedy loop is
//             exact integer arithmetic: the picks do not depend on any summation order, and
//             mathematically tied candidates (common: two tokens that only improve each other's
//             coverage) are exact ties that go to the lowest index.
//   k_greedy  one workgroup per (sample, region); the region's whole S (up to 256 x 256 words)
//             lives in the workgroup's vector registers (see the comment at the kernel).
#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

// Similarities are decided on a grid of 2^-22: |S| <= 1, so a 256-term sum of differences
// max(0, S_ij - m_j) <= 2^23 stays below 2^31 and is exact in a 32-bit integer.
constexpr double kSimScale = 4194304.0;

// ------------------------------------------------------------------------------------------------
// 64 x 64 block of one region's similarity matrix per workgroup, 2 x 2 waves of 32 x 32.  S is
// symmetric: only blocks on or above the diagonal are computed and each value is stored twice.
// The token norms come out of the same pass: while a K slice sits in LDS, the first 128 threads add
// the squares of one row each (64 rows of the left operand, 64 of the right) in double.
template <typename T>
__global__ __launch_bounds__(256) void k_gram(const T *__restrict__ X, int32_t *__restrict__ S, RegionMap map,
                                             int N, int C, int P, int n_loc, int tiles) {
  constexpr int BK = 32;
  constexpr int EPP = 16 / (int)sizeof(T);
  constexpr int LDK = BK + EPP;
  constexpr int PPR = BK / EPP;
  constexpr int NP = 64 * PPR / 256;
  __shared__ __align__(16) T As[64 * LDK];
  __shared__ __align__(16) T Bs[64 * LDK];
  __shared__ double nrm[128];

  // blockIdx.x enumerates the pairs (tm <= tn) row by row
  int tm = 0, rest = blockIdx.x;
  while (rest >= tiles - tm) { rest -= tiles - tm; tm++; }
  const int tn = tm + rest;
  const int bp = blockIdx.y, b = bp / P, p = bp % P;
  const int m0 = tm * 64, n0 = tn * 64;
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
  double sq = 0.0;
  const T *my_row = tid < 64 ? As + tid * LDK : Bs + (tid - 64) * LDK;

  Pkt ra[NP], rb[NP];
#pragma unroll
  for (int i = 0; i < NP; i++) {
    ra[i] = pa[i] ? pkt_load(pa[i]) : pkt_zero();
    rb[i] = pb[i] ? pkt_load(pb[i]) : pkt_zero();
  }
  for (int k0 = 0; k0 < C; k0 += BK) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NP; i++) {
      pkt_store(As + lo[i], ra[i]);
      pkt_store(Bs + lo[i], rb[i]);
    }
    __syncthreads();
    if (k0 + BK < C) {
#pragma unroll
      for (int i = 0; i < NP; i++) {
        ra[i] = pa[i] ? pkt_load(pa[i] + k0 + BK) : pkt_zero();
        rb[i] = pb[i] ? pkt_load(pb[i] + k0 + BK) : pkt_zero();
      }
    }
    if (tid < 128) {
#pragma unroll
      for (int k = 0; k < BK; k++) {
        double v = (double)to_f32(my_row[k]);
        sq += v * v;
      }
    }
    Frag<T> fa[2], fb[2];
#pragma unroll
    for (int i = 0; i < 2; i++) {
      frag_load_kc(fa[i], As + (wm * 32 + 16 * i + c) * LDK + 8 * g);
      frag_load_kc(fb[i], Bs + (wn * 32 + 16 * i + c) * LDK + 8 * g);
    }
#pragma unroll
    for (int s8 = 0; s8 < 8; s8++)
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)to_f32(fa[i].v[s8]), (double)to_f32(fb[j].v[s8]),
                                                           acc[i][j], 0, 0, 0);
  }
  if (tid < 128) {
    double n = sqrt(sq);
    nrm[tid] = n > 1e-12 ? n : 1e-12;
  }
  __syncthreads();

  // fp64 accumulator tile: lane holds column lane % 16 and rows (lane / 16) + 4 r.
  int32_t *Sr = S + (size_t)bp * n_loc * n_loc;
#pragma unroll
  for (int j = 0; j < 2; j++) {
    int cl = wn * 32 + 16 * j + c, col = n0 + cl;
    if (col >= n_loc) continue;
    double ncol = nrm[64 + cl];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        int rl = wm * 32 + 16 * i + g + 4 * r, row = m0 + rl;
        if (row < n_loc) {
          int32_t v = (int32_t)rint(acc[i][j][r] / (nrm[rl] * ncol) * kSimScale);
          Sr[(size_t)row * n_loc + col] = v;
          if (tm != tn) Sr[(size_t)col * n_loc + row] = v;
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------
// Greedy facility location, one workgroup per (sample, region), exact and lazy.
//
// Arithmetic.  S is on a grid of 2^-22 (kSimScale): a term max(0, S_ij - m_j) is at most 2^23 and a
// 256-term sum fits an unsigned 32-bit register, so values, sums and comparisons are plain 32-bit
// integer instructions and every cross-lane step is a single DPP-modified add or max.
// Layout.  Wave w owns rows 32w .. 32w+31 of the region's S; lane l holds, of each of those rows,
// the columns l + 64u.  Evaluating one row's value is a few integer operations per lane plus one
// 64-lane reduction, and WHICH rows are evaluated is a wave-uniform (scalar) decision.
// Keys.  Lane r < 32 of wave w keeps key = value + 1 of row 32w + r (0 = chosen or absent).
// Across waves a candidate travels as (key << 8) | (255 - row): the largest packed word is the
// largest value and, among equals, the lowest index, so the workgroup's argmax is one LDS
// atomic max per wave.
// Laziness.  Values only shrink as m grows (diminishing returns, paper Sec. 3.2), so a key from an
// earlier round is an upper bound.  In a round every wave re-evaluates its row with the largest
// stale key and posts that fresh candidate together with the best of its remaining stale keys.
// If no stale key in the workgroup beats the best fresh candidate B0, B0 is the pick (one barrier
// per round, the common case).  Otherwise every wave re-evaluates exactly its rows whose stale key
// still beats B0 and the waves vote again.  Rows that are skipped cannot win, so the pick is the
// one a full rescan (Alg. 2) makes.
// ------------------------------------------------------------------------------------------------
template <int CTRL, int ROW_MASK = 0xf> __device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppRor4 = 0x124, kDppRor8 = 0x128;
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;

// sum over the 64 lanes (mod 2^32); the result is uniform
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  v += dpp_u32<kDppXor1>(v);
  v += dpp_u32<kDppXor2>(v);
  v += dpp_u32<kDppRor4>(v);
  v += dpp_u32<kDppRor8>(v);               // every lane: total of its row of 16
  v += dpp_u32<kDppBcast15, 0xa>(v);       // rows 1, 3 += rows 0, 2
  v += dpp_u32<kDppBcast31, 0xc>(v);       // rows 2, 3 += rows 0 + 1
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
// max over lanes 0..31; the result is uniform
__device__ __forceinline__ uint32_t wave_max32_u32(uint32_t v) {
  v = max(v, dpp_u32<kDppXor1>(v));
  v = max(v, dpp_u32<kDppXor2>(v));
  v = max(v, dpp_u32<kDppRor4>(v));
  v = max(v, dpp_u32<kDppRor8>(v));
  return max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16));
}

#ifndef TOMA_GREEDY_TOPK
#define TOMA_GREEDY_TOPK 2
#endif
template <int NT>
__global__ __launch_bounds__(64 * ((NT + 1) / 2)) void k_greedy(const int32_t *__restrict__ S,
                                                             int32_t *__restrict__ idx,
                                                             float *__restrict__ gain_out, RegionMap map,
                                                             int P, int d_loc) {
  constexpr int NL = 16 * NT;          // tokens in the region
  constexpr int NW = (NT + 1) / 2;     // waves, 32 rows each
  constexpr int CPL = (NT + 3) / 4;    // columns per lane
  constexpr int32_t kPad = 1 << 23;    // m of a padding column: above every S, so it never contributes
  constexpr uint32_t kBias0 = 1u << 30;  // first step: row sums are signed, |sum| <= 2^30
  constexpr int kBulk = 12;            // refresh all rows at once when at least this many are due
  constexpr int kTopK = TOMA_GREEDY_TOPK;  // keys per wave that phase 1 refreshes
  __shared__ int32_t rowbuf[2][NW][64 * CPL];   // [round parity]: each wave's candidate row
  // packed best candidates, rotated over three rounds so that a slot is cleared two rounds
  // before it is written again: [round % 3][0 fresh, 1 best stale runner-up, 2 after phase 2]
  __shared__ __align__(16) unsigned long long slot[3][4];

  const int bp = blockIdx.x, p = bp % P;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int32_t *Sr = S + (size_t)bp * NL * NL;

  // sv[u][r]: column lane + 64 u of row 32 w + r.  One 32-wide register vector per u, so that a
  // wave-uniform row number r indexes the registers directly (relative addressing), no dispatch.
  typedef int32_t i32x32 __attribute__((ext_vector_type(32)));
  i32x32 sv[CPL];
  int32_t m[CPL];
  bool col_ok[CPL];
#pragma unroll
  for (int u = 0; u < CPL; u++) {
    col_ok[u] = lane + 64 * u < NL;
    m[u] = kPad;
  }
#pragma unroll
  for (int r = 0; r < 32; r++)
#pragma unroll
    for (int u = 0; u < CPL; u++) {
      int row = 32 * w + r;
      sv[u][r] = (row < NL && col_ok[u]) ? Sr[(size_t)row * NL + lane + 64 * u] : 0;
    }
  int32_t msum = 0;  // sum of this lane's m: sum_u max(0, s - m) = sum_u max(s, m) - msum

  const int my_row = 32 * w + lane;
  const bool my_live0 = lane < 32 && my_row < NL;
  uint32_t key = 0;  // lane r < 32: value + 1 of row 32w + r, an upper bound between refreshes

  // value of row r of this wave (r is wave-uniform): first step = row sum, later = sum max(0, S - m)
  auto eval = [&](int r, bool first) -> uint32_t {
    int32_t part = first ? 0 : -msum;
#pragma unroll
    for (int u = 0; u < CPL; u++) {
      const int32_t v = sv[u][r];
      part += first ? v : max(v, m[u]);
    }
    return wave_sum_u32((uint32_t)part);
  };
  // the same, and the row is also posted to rowbuf[buf][w]
  auto eval_post = [&](int buf, int r) -> uint32_t {
    int32_t part = -msum;
#pragma unroll
    for (int u = 0; u < CPL; u++) {
      const int32_t v = sv[u][r];
      part += max(v, m[u]);
      rowbuf[buf][w][lane + 64 * u] = v;
    }
    return wave_sum_u32((uint32_t)part);
  };
  // refresh the keys of all live rows of this wave at once (straight-line code, independent chains)
  auto eval_all = [&](bool first) {
#pragma unroll
    for (int r = 0; r < 32; r++) {
      int32_t part = first ? 0 : -msum;
#pragma unroll
      for (int u = 0; u < CPL; u++) part += first ? sv[u][r] : max(sv[u][r], m[u]);
      uint32_t g = wave_sum_u32((uint32_t)part);
      if (lane == r && (first ? my_live0 : key != 0)) key = g + 1u + (first ? kBias0 : 0u);
    }
  };
  auto post_row = [&](int buf, int r) {
#pragma unroll
    for (int u = 0; u < CPL; u++) rowbuf[buf][w][lane + 64 * u] = sv[u][r];
  };
  // slots 0 and 1 of a round in one 16-byte LDS read
  auto read_slots = [&](const unsigned long long *ptr, unsigned long long &a, unsigned long long &b) {
    const u32x4 v = *reinterpret_cast<const u32x4 *>(ptr);
    const uint32_t a0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)v[0]);
    const uint32_t a1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)v[1]);
    const uint32_t b0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)v[2]);
    const uint32_t b1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)v[3]);
    a = ((unsigned long long)a1 << 32) | a0;
    b = ((unsigned long long)b1 << 32) | b0;
  };
  auto read_slot = [&](const unsigned long long *ptr) -> unsigned long long {
    unsigned long long v = *ptr;
    uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
  };
  // one LDS atomic from the calling lane (no wave-wide combining code around it)
  auto lds_max_u64 = [&](unsigned long long *ptr, unsigned long long v) {
    const uint32_t addr = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)ptr;
    asm volatile("ds_max_u64 %0, %1" ::"v"(addr), "v"(v) : "memory");
  };
  auto pack = [&](uint32_t k, int r) -> unsigned long long {
    return ((unsigned long long)k << 8) | (unsigned)(255 - (32 * w + r));
  };

  // LDS traffic is the only thing the waves exchange inside the loop: wait for it, then meet
  auto lds_barrier = [&]() {
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
  // picks and their values are kept in registers of wave 0 (pick k in lane k % 64) and written
  // once at the end, so that no global store sits on the loop's critical path
  int32_t pick_row[CPL];
  uint32_t pick_key[CPL];
#pragma unroll
  for (int u = 0; u < CPL; u++) { pick_row[u] = 0; pick_key[u] = 0; }

  if (threadIdx.x < 12) slot[threadIdx.x / 4][threadIdx.x % 4] = 0;
  lds_barrier();

  int q3 = 0;  // step % 3
  for (int step = 0; step < d_loc; step++) {
    const bool first = step == 0;
    const int buf = step & 1;
    unsigned long long *sl = slot[q3];
    bool fresh = false;
    // ---- phase 1: refresh the row with the largest stale key; post it, and the best of the rest ----
    if (first) {
      eval_all(true);
      fresh = true;
    }
    {
      const uint32_t top = wave_max32_u32(key);
      if (top != 0) {
        const int r1 = __builtin_ctzll(__ballot(key == top && lane < 32));
        if (first) {
          post_row(buf, r1);
          if (lane == 0) lds_max_u64(&sl[0], pack(top, r1));
        } else if (kTopK > 1) {
          // the kTopK largest keys are refreshed together (independent chains); the best of the
          // remaining keys stays a stale bound
          uint32_t kk = key, tk[kTopK];
          int rk[kTopK];
          tk[0] = top; rk[0] = r1;
#pragma unroll
          for (int i = 1; i < kTopK; i++) {
            kk = lane == rk[i - 1] ? 0u : kk;
            tk[i] = tk[i - 1] ? wave_max32_u32(kk) : 0u;
            rk[i] = tk[i] ? __builtin_ctzll(__ballot(kk == tk[i] && lane < 32)) : rk[0];
          }
          kk = lane == rk[kTopK - 1] ? 0u : kk;
          const uint32_t rest = tk[kTopK - 1] ? wave_max32_u32(kk) : 0u;
          const unsigned long long rest_lanes = __ballot(kk == rest && lane < 32);
          uint32_t gk[kTopK];
#pragma unroll
          for (int i = 0; i < kTopK; i++) gk[i] = tk[i] ? eval(rk[i], false) + 1u : 0u;
          uint32_t gc = gk[0];
          int rc = rk[0];
          fresh = lane == rk[0];
          key = lane == rk[0] ? gk[0] : key;
#pragma unroll
          for (int i = 1; i < kTopK; i++) {
            if (tk[i]) {
              key = lane == rk[i] ? gk[i] : key;
              fresh = fresh || lane == rk[i];
              if (gk[i] > gc || (gk[i] == gc && rk[i] < rc)) { gc = gk[i]; rc = rk[i]; }
            }
          }
          post_row(buf, rc);
          if (lane == 0) {
            lds_max_u64(&sl[0], pack(gc, rc));
            if (rest != 0) lds_max_u64(&sl[1], pack(rest, __builtin_ctzll(rest_lanes)));
          }
        } else {
          // the best of the other keys stays a stale bound (independent of the refresh below)
          const uint32_t k2 = lane == r1 ? 0u : key;
          const uint32_t rest = wave_max32_u32(k2);
          const unsigned long long rest_lanes = __ballot(k2 == rest && lane < 32);
          const uint32_t g = eval_post(buf, r1) + 1u;
          const bool mine = lane == r1;
          key = mine ? g : key;
          fresh = mine;
          if (lane == 0) {
            lds_max_u64(&sl[0], pack(g, r1));
            if (rest != 0) lds_max_u64(&sl[1], pack(rest, __builtin_ctzll(rest_lanes)));
          }
        }
      }
    }
    lds_barrier();
    if (threadIdx.x < 4) slot[q3 == 0 ? 2 : q3 - 1][threadIdx.x] = 0;  // the slots of round step + 2
    unsigned long long best, stale;
    read_slots(sl, best, stale);
    if (!first) {
      if (stale > best) {
        // ---- phase 2: some stale key still beats the best fresh candidate: refresh those rows ----
        uint32_t g0 = (uint32_t)(best >> 8);
        int i0 = 255 - (int)(best & 255u);
        bool beats = key > g0 || (key == g0 && my_row < i0);
        unsigned long long need = __ballot(key != 0 && !fresh && beats && lane < 32);
        if (__builtin_popcountll(need) >= kBulk) {
          eval_all(false);
        } else {
          // two rows per turn: their reduction chains are independent and interleave
          while (need) {
            const int ra = __builtin_ctzll(need);
            need &= need - 1;
            const int rb = need ? __builtin_ctzll(need) : ra;
            need &= need - 1;
            const uint32_t ga = eval(ra, false) + 1u, gb = eval(rb, false) + 1u;
            key = lane == ra ? ga : key;
            key = lane == rb ? gb : key;
          }
        }
        uint32_t top = wave_max32_u32(key);
        if (top != 0) {
          int r = __builtin_ctzll(__ballot(key == top && lane < 32));
          post_row(buf, r);
          if (lane == 0) lds_max_u64(&sl[2], pack(top, r));
        }
        lds_barrier();
        best = read_slot(&sl[2]);
      }
    }
    const uint32_t G = (uint32_t)(best >> 8);
    const int I = 255 - (int)(best & 255u);
    const int ww = I >> 5;
    msum = 0;
#pragma unroll
    for (int u = 0; u < CPL; u++) {
      int32_t mv = rowbuf[buf][ww][lane + 64 * u];
      m[u] = !col_ok[u] ? kPad : (first ? mv : max(m[u], mv));
      msum += m[u];
    }
    if (first && my_live0) key = 0xffffffffu;  // row sums are no bounds on later values: force a refresh
    key = (w == ww && lane == (I & 31)) ? 0u : key;
#pragma unroll
    for (int u = 0; u < CPL; u++) {
      const bool here = step == lane + 64 * u;
      pick_row[u] = here ? I : pick_row[u];
      pick_key[u] = here ? G : pick_key[u];
    }
    q3 = q3 == 2 ? 0 : q3 + 1;
  }
  if (w == 0) {
#pragma unroll
    for (int u = 0; u < CPL; u++) {
      const int k = lane + 64 * u;
      if (k < d_loc) {
        idx[(size_t)bp * d_loc + k] = map.token(p, pick_row[u]);
        const double v = (double)pick_key[u] - 1.0 - (k == 0 ? (double)kBias0 : 0.0);
        if (gain_out) gain_out[(size_t)bp * d_loc + k] = (float)(v / kSimScale);
      }
    }
  }
}

template <typename T>
static int select_typed(const Shape &s, const T *X, int32_t *idx, float *gain, char *ws, const Workspace &w,
                        hipStream_t st) {
  int32_t *S = reinterpret_cast<int32_t *>(ws + w.sim);
  RegionMap map{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  int tiles = (s.n_loc + 63) / 64;
  { KernelTimer kt(K_GRAM, st);
  hipLaunchKernelGGL(k_gram<T>, dim3(tiles * (tiles + 1) / 2, s.B * s.P), dim3(256), 0, st, X, S, map, s.N, s.C,
                     s.P, s.n_loc, tiles); }
  int regions = s.B * s.P;
  KernelTimer kt(K_GREEDY, st);
  switch (s.n_loc / 16) {
#define TOMA_GREEDY_CASE(NT)                                                                              \
  case NT:                                                                                                \
    hipLaunchKernelGGL(k_greedy<NT>, dim3(regions), dim3(64 * ((NT + 1) / 2)), 0, st, S, idx, gain, map, s.P, \
                       s.d_loc);                                                                           \
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
