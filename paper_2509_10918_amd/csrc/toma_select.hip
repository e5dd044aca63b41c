// Destination selection: cosine similarity inside each region and the greedy facility-location
// pick sequence (paper Sec. 4.1, Eq. 2, Alg. 2; regions as in Alg. 3 step 1).
//
// Two kernels:
//   k_gram    S = cos(x_i, x_j) per region with the fp64 matrix cores (v_mfma_f64_16x16x4_f64):
//             products of stored bf16 / fp32 values are exact in double, so S is the similarity
//             to ~1e-16 before it is rounded once to the nearest multiple of 2^-30 and stored as
//             a 32-bit integer.  From there on every sum and comparison of the greedy loop is
//             exact integer arithmetic: the picks do not depend on any summation order, and
//             mathematically tied candidates (common: two tokens that only improve each other's
//             coverage) are exact ties that go to the lowest index.
//   k_greedy  one workgroup per (sample, region); the region's whole S (up to 256 x 256 words)
//             lives in the workgroup's vector registers and the rows' values are kept up to date
//             incrementally (see the comment at the kernel).
#include <type_traits>

#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

// Similarities are decided on a grid of 2^-30: |S| <= 1 fits a 32-bit integer, a difference
// max(0, S_ij - m_j) <= 2^31 an unsigned one, and sums of up to 256 of them are kept in 64 bits.
// The grid is what makes mathematically tied candidates exact ties; it is fine enough that
// rounding to it does not decide between candidates that are not tied (a row's value moves by at
// most 2^-31 per term, below 1e-6 of any value above 2.4e-4 even with all 256 terms adverse).
constexpr double kSimScale = 1073741824.0;

// ------------------------------------------------------------------------------------------------
// One wave per 16 x 16 block of one region's similarity matrix.  S is symmetric: only blocks on or
// above the diagonal are computed and each value is stored twice.
// The fp64 matrix cores are slow enough (one 16 x 16 x 4 product keeps them busy for tens of
// cycles) that operand traffic does not matter: every lane reads its fragments straight from global
// memory (row = lane % 16, eight consecutive channels of k-group lane / 16 per 32-channel chunk), no
// LDS and no barrier, two chunks ahead of the products; small independent units spread evenly over
// the chip's SIMDs, which is what bounds this kernel.  The token norms come out of the same pass
// (sums of squares of the values a lane holds anyway, combined across the four k-groups).
template <typename T, int KS>
__global__ __launch_bounds__(256) void k_gram(const T *__restrict__ X, int32_t *__restrict__ S, RegionMap map,
                                             int N, int C, int P, int n_loc, int tiles, int units) {
  constexpr int EPP = 16 / (int)sizeof(T);  // elements per 16-byte packet
  constexpr int NPK = 8 / EPP;              // packets per fragment (eight channels)
  constexpr int UPW = 4 / KS;               // units per workgroup: KS waves share one, each a slice of K
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  // one-dimensional grid over (region, group of UPW units), remapped so that an XCD works on whole
  // regions: their tokens then stay in that XCD's L2
  const int groups = (units + UPW - 1) / UPW;
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  const int bp = work / groups;
  const int unit_raw = (work - bp * groups) * UPW + w / KS, kh = w % KS;
  const bool live = unit_raw < units;
  const int unit = live ? unit_raw : units - 1;
  // unit enumerates the pairs (tm <= tn) row by row
  int tm = 0, rest = unit;
  while (rest >= tiles - tm) { rest -= tiles - tm; tm++; }
  const int tn = tm + rest;
  const int b = bp / P, p = bp % P;
  const int nchunk_all = C / 32;
  const int c_lo = nchunk_all * kh / KS, nchunk = live ? nchunk_all * (kh + 1) / KS - c_lo : 0;
  const T *Xb = X + (size_t)b * N * C + 32 * c_lo;
  const T *pa = Xb + (size_t)map.token(p, 16 * tm + c) * C + 8 * g;
  const T *pb = Xb + (size_t)map.token(p, 16 * tn + c) * C + 8 * g;

  struct Chunk { Pkt a[NPK], b[NPK]; };
  auto fetch = [&](Chunk &ch, int k0) {
#pragma unroll
    for (int i = 0; i < NPK; i++) {
      ch.a[i] = pkt_load(pa + k0 + i * EPP);
      ch.b[i] = pkt_load(pb + k0 + i * EPP);
    }
  };
  auto value = [&](const Pkt (&pk)[NPK], int s8) -> double {
    if constexpr (sizeof(T) == 2) {
      // bf16 -> fp32 is a 16-bit shift
      const u32x4 q = pk[0].v;
      const uint32_t word = q[s8 >> 1];
      return (double)__builtin_bit_cast(float, (s8 & 1) ? (word & 0xffff0000u) : (word << 16));
    } else {
      const u32x4 q = pk[s8 >> 2].v;
      const uint32_t word = q[s8 & 3];
      return (double)__builtin_bit_cast(float, word);
    }
  };

  // two accumulators: consecutive products do not wait for each other
  f64x4 acc = (f64x4){0.0, 0.0, 0.0, 0.0}, acc1 = (f64x4){0.0, 0.0, 0.0, 0.0};
  double sqa = 0.0, sqb = 0.0;
  Chunk c0, c1, c2;
  if (nchunk > 0) fetch(c0, 0);
  if (nchunk > 1) fetch(c1, 32);
  for (int i = 0; i < nchunk; i += 3) {
    // three-deep rotation written out so that the buffers stay in registers
    auto work = [&](Chunk &cur, Chunk &nxt2, int ii) {
      if (ii + 2 < nchunk) fetch(nxt2, (ii + 2) * 32);
#pragma unroll
      for (int s8 = 0; s8 < 8; s8++) {
        const double av = value(cur.a, s8), bv = value(cur.b, s8);
        sqa += av * av;
        sqb += bv * bv;
        if (s8 & 1) acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc1, 0, 0, 0);
        else acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
      }
    };
    work(c0, c2, i);
    if (i + 1 < nchunk) work(c1, c0, i + 1);
    if (i + 2 < nchunk) work(c2, c1, i + 2);
  }
  acc += acc1;
  if constexpr (KS > 1) {
    // the waves of a unit add their slices of K up in the first of them
    __shared__ double part[4][6][64];
    if (kh != 0) {
#pragma unroll
      for (int r = 0; r < 4; r++) part[w][r][lane] = acc[r];
      part[w][4][lane] = sqa;
      part[w][5][lane] = sqb;
    }
    __syncthreads();
    if (kh != 0 || !live) return;
#pragma unroll
    for (int o = 1; o < KS; o++) {
#pragma unroll
      for (int r = 0; r < 4; r++) acc[r] += part[w + o][r][lane];
      sqa += part[w + o][4][lane];
      sqb += part[w + o][5][lane];
    }
  } else {
    if (!live) return;
  }
  // norms of row 16 tm + c and of row 16 tn + c: sum over the four k-groups
  sqa += wave_xor_f64(sqa, 16); sqa += wave_xor_f64(sqa, 32);
  sqb += wave_xor_f64(sqb, 16); sqb += wave_xor_f64(sqb, 32);
  double na = sqrt(sqa), nb = sqrt(sqb);
  na = na > 1e-12 ? na : 1e-12;
  nb = nb > 1e-12 ? nb : 1e-12;

  // fp64 accumulator tile: lane holds column lane % 16 and rows (lane / 16) + 4 r.
  int32_t *Sr = S + (size_t)bp * n_loc * n_loc;
  const int col = 16 * tn + c;
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int rl = g + 4 * r, row = 16 * tm + rl;
    const double nrow = __shfl(na, rl, 64);
    const int32_t v = (int32_t)rint(acc[r] / (nrow * nb) * kSimScale);
    Sr[(size_t)row * n_loc + col] = v;
    if (tm != tn) Sr[(size_t)col * n_loc + row] = v;
  }
}

// ------------------------------------------------------------------------------------------------
// Greedy facility location, one workgroup per (sample, region): exact, with incremental gains.
//
// Arithmetic.  S is on a grid of 2^-30 (kSimScale) and fits a 32-bit register; a term
// max(0, S_ij - m_j) is at most 2^31 and a 256-term sum at most 2^39, so the rows' values are 64-bit
// integers: values, sums and comparisons are plain integer instructions, independent of any
// summation order.  Only the first rounds have values of 4 or more; the rest run on 32-bit words.
// Incremental gains.  After a pick t only the columns j with S_tj > m_j change their coverage, and
// the value of row i drops by exactly  sum over those j of  med(S_ij, m_j, m_j') - m_j  (m' the new
// coverage).  Because the arithmetic is exact, subtracting these differences keeps every row's value
// equal to the full rescan sum_j max(0, S_ij - m_j) of Alg. 2, at a cost proportional to the number
// of changed columns (a handful per round once a few destinations exist) instead of N_loc^2.
// The first pick (largest row sum) is the same rule started from the coverage m = -1 everywhere:
// sum_j max(0, S_ij + 1) = row sum + N_loc, so the loop has no special first round.
// Layout.  With NW waves, every wave owns one of each NW consecutive columns of S, for ALL rows, in
// its register c = column / NW (c < 32) - which one rotates from tile row to tile row, so that the
// columns that tend to change together, a pick's neighbours along and across the tile's rows, are
// spread over the waves; lane l holds the rows RPL l + v, sv[v][c] = S[RPL l + v][column of
// register c] (128 registers for a 256-token region).  The
// coverage of the own columns lives in lanes 0..31.  A changed column costs its owner a few
// instructions with the column's (m, m') as scalar operands and the column's registers addressed
// relative to the wave-uniform column number (scalar branches cost far more here than indexing).
// Exchange, two barriers per round.  The rows' comparison keys (value + 1; 0 = picked or absent)
// live in LDS.  (1) Every wave reads all keys (RPL per lane) and finds the same argmax t on its own
// (the high words first, then the low words of the rows that hold the largest high word: two DPP
// reductions and a ballot; lanes are in row order, so the lowest lane among equals holds the lowest
// index).  By symmetry the owner of column t holds the whole row t, one word per (lane, v): it posts
// the row to LDS, ordered so that every wave then reads its own columns as one contiguous run.
// Barrier.  (2) Each wave subtracts its rows' decreases from the keys with integer LDS atomics (they
// commute, so the result does not depend on their order).  A picked row's value falls to exactly
// zero with its own pick's decrease; one more atomic takes away the + 1, which leaves key 0 for
// good.  Barrier.
// GAP: wave 0 also finds the largest key among the rows other than the pick (the runner-up) and
// records the difference; the other waves skip it.
// ------------------------------------------------------------------------------------------------
template <int CTRL, int ROW_MASK = 0xf> __device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppRor4 = 0x124, kDppRor8 = 0x128;

// max over the 64 lanes; the result is uniform
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, dpp_u32<kDppXor1>(v));
  v = max(v, dpp_u32<kDppXor2>(v));
  v = max(v, dpp_u32<kDppRor4>(v));
  v = max(v, dpp_u32<kDppRor8>(v));  // every lane: maximum of its row of 16
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return max(max(a, b), max(c, d));
}
// max over the 64 lanes of 64-bit keys: the largest high word, then the largest low word among its
// holders; the result is uniform
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t k) {
  const uint32_t hi = (uint32_t)(k >> 32), lo = (uint32_t)k;
  const uint32_t top_hi = wave_max_u32(hi);
  const uint32_t top_lo = wave_max_u32(hi == top_hi ? lo : 0u);
  return ((uint64_t)top_hi << 32) | top_lo;
}

// What the selection kernel needs to recompute flagged rows of S in double precision (flag == null: none).
struct RowFix { const bf16_t *X; const double *nrm; const uint8_t *flag; int N, C; };

constexpr uint64_t kNoRunnerUp = ~0ull;  // recorded gap when the pick was the last candidate

// CLOCKS (a profiling aid, never the product's kernel): every wave also adds up the shader clocks it
// spends in each part of a round and leaves the sums in clk_out[(region * NW + wave) * 8 + ...]:
// 0 keys read and argmax, 1 row t posted and first barrier, 2 own columns read and the changed ones
// found, 3 changed columns and atomics, 4 second barrier; 5 rounds, 6 changed columns this wave owned.
template <int NT, bool GAP, bool CLOCKS = false>
__global__ __launch_bounds__(64 * ((NT + 1) / 2)) void k_greedy(int32_t *S, int32_t *__restrict__ idx,
                                                             float *__restrict__ gain_out,
                                                             float *__restrict__ gap_out, RegionMap map,
                                                             int P, int d_loc, RowFix fix,
                                                             unsigned long long *__restrict__ clk_out) {
  constexpr int NL = 16 * NT;          // tokens in the region
  constexpr int NW = (NT + 1) / 2;     // waves, up to 32 columns each
  constexpr int RPL = (NL + 63) / 64;  // rows per lane: lane l holds rows RPL l .. RPL l + RPL - 1
  constexpr int32_t kPad = (1 << 30) + 1;  // coverage of a padding column: above every S, so it never changes
  constexpr int32_t kFloor = -(1 << 30);   // similarity -1: the coverage before the first pick
  __shared__ uint64_t keys[RPL * 64];      // [64 v + l]: value + 1 of row RPL l + v, 0 once picked
  __shared__ uint32_t keys32[RPL * 64];    // the same once every key fits 32 bits
  __shared__ int32_t rowt[NW * 32];        // row t: wave w's column of register c at [32 w + c]
  __shared__ int32_t pick_row[RPL * 64];   // row of every pick
  __shared__ uint64_t pick_val[RPL * 64];  // its value
  __shared__ uint64_t pick_gap[GAP ? RPL * 64 : 1];  // its lead over the runner-up

  const int bp = blockIdx.x, p = bp % P;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, cl = lane & 31;
  int32_t *Sr = S + (size_t)bp * NL * NL;

  // Rows of S that the fixed-point similarity kernel could not do exactly (a token with more than a few
  // elements far below its largest, flag 2: very rare) are recomputed here in double precision, before
  // anything reads them.
  if (fix.flag) {
    const size_t tok0 = (size_t)(bp / P) * fix.N;
    // (the flags of the region's tokens, one bit each, gathered once: keys[] is free until the rounds start)
    uint32_t *fbits = reinterpret_cast<uint32_t *>(keys);
    for (int l = threadIdx.x; l < 8; l += 64 * NW) fbits[l] = 0u;
    __syncthreads();
    int mine = 0;
    for (int l = threadIdx.x; l < NL; l += 64 * NW)
      if (fix.flag[tok0 + map.token(p, l)] == 2) { mine = 1; atomicOr(&fbits[l >> 5], 1u << (l & 31)); }
    if (__syncthreads_or(mine)) {
      for (int t = 0; t < NL; t++) {
        if (!((fbits[t >> 5] >> (t & 31)) & 1u)) continue;  // (uniform)
        const size_t tt = tok0 + map.token(p, t);
        const bf16_t *xt = fix.X + tt * fix.C;
        // a wave per partner token, its lanes across the channels (eight each per step)
        for (int j = w; j < NL; j += NW) {
          const size_t tj = tok0 + map.token(p, j);
          const bf16_t *xj = fix.X + tj * fix.C;
          double dot = 0.0;
          for (int ch = 8 * lane; ch < fix.C; ch += 512) {
            const Pkt pa = pkt_load(xt + ch), pb = pkt_load(xj + ch);
#pragma unroll
            for (int u = 0; u < 4; u++) {
              const uint32_t wa = pa.v[u], wb = pb.v[u];
              dot += (double)__builtin_bit_cast(float, wa << 16) * (double)__builtin_bit_cast(float, wb << 16);
              dot += (double)__builtin_bit_cast(float, wa & 0xffff0000u) * (double)__builtin_bit_cast(float, wb & 0xffff0000u);
            }
          }
#pragma unroll
          for (int msk = 1; msk < 64; msk <<= 1) dot += wave_xor_f64(dot, msk);
          if (lane == 0) {
            const int32_t v = (int32_t)rint(dot / (fix.nrm[tt] * fix.nrm[tj]) * kSimScale);
            Sr[(size_t)t * NL + j] = v;
            Sr[(size_t)j * NL + t] = v;
          }
        }
      }
      __threadfence();
      __syncthreads();
    }
  }

  // Which wave owns which column.  Of every NW consecutive columns each wave owns one, kept in its
  // register c = column / NW; plainly, wave w would own the columns congruent to w.  A pick raises the
  // coverage of the tokens around it in the tile, and tokens above one another are tile_w columns apart - a
  // multiple of NW for the usual tiles, so whole vertical runs would fall to one wave, which then
  // applies them one after the other while the rest wait.  Where the tile's width allows it (a power of
  // two and a multiple of NW) the assignment is therefore rotated by three from one tile row to the next.
  const int tile_w = map.tile_w;
  const bool skewed = (tile_w & (tile_w - 1)) == 0 && tile_w % NW == 0 && NL % NW == 0;
  const int skew = skewed ? 3 : 0, tw_sh = skewed ? __builtin_ctz(tile_w) : 0;
  auto wave_of = [&](int col) { return (col + skew * (col >> tw_sh)) % NW; };
  auto col_of = [&](int c) {  // the column this wave keeps in register c
    const int base = NW * c;
    return base + ((w - skew * (base >> tw_sh)) % NW + NW) % NW;
  };
  // Loaded through the symmetric element S[column][RPL l + v]: a lane reads RPL consecutive
  // words and consecutive lanes continue the run.
  typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
  typedef int32_t i32x32 __attribute__((ext_vector_type(32)));
  i32x32 sv[RPL];  // register vectors, indexed by wave-uniform column numbers (relative addressing)
#pragma unroll
  for (int c = 0; c < 32; c++) {
    const int col = col_of(c);
    if constexpr (RPL == 4) {  // NL is a multiple of 16: the four rows of a lane exist together
      const bool ok = col < NL && 4 * lane < NL;
      const i32x4 q = ok ? *reinterpret_cast<const i32x4 *>(Sr + (size_t)col * NL + 4 * lane) : (i32x4){0, 0, 0, 0};
      sv[0][c] = q[0]; sv[1][c] = q[1]; sv[2][c] = q[2]; sv[3][c] = q[3];
    } else {
#pragma unroll
      for (int v = 0; v < RPL; v++) {
        const int row = RPL * lane + v;
        sv[v][c] = (col < NL && row < NL) ? Sr[(size_t)col * NL + row] : 0;
      }
    }
  }
  // this lane keeps the coverage of the column of register cl (lanes l and l + 32 hold the same; only
  // the first 32 report changes, and never for a column past the region's end)
  const bool col_ok = col_of(cl) < NL, reports = col_ok && lane < 32;
  int32_t m = col_ok ? kFloor : kPad;
  // where this lane's rows go in rowt (as columns, by symmetry)
  int post_at[RPL];
#pragma unroll
  for (int v = 0; v < RPL; v++) {
    const int j = RPL * lane + v;
    post_at[v] = j < NL ? wave_of(j) * 32 + j / NW : -1;
  }

  auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  // keys under the starting coverage: 1 + sum_j (S_ij + 1); the slots of row t that stand for
  // columns past the region's end are never posted: they start, and stay, at zero
  for (int i = threadIdx.x; i < RPL * 64; i += 64 * NW) keys[i] = RPL * (i & 63) + (i >> 6) < NL ? 1u : 0u;
  for (int i = threadIdx.x; i < NW * 32; i += 64 * NW) rowt[i] = 0;
  lds_barrier();
#pragma unroll
  for (int v = 0; v < RPL; v++) {
    uint64_t part = 0;
#pragma unroll
    for (int c = 0; c < 32; c++)
      if (col_of(c) < NL) part += (uint32_t)(sv[v][c] - kFloor);
    if (RPL * lane + v < NL)
      __hip_atomic_fetch_add(&keys[64 * v + lane], part, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  lds_barrier();

  // One round, with the keys as 64-bit (WIDE) or 32-bit words.  The winning value never grows from
  // one round to the next (diminishing returns), so once the largest key fits 32 bits every key does
  // for good, and no row's decrease in a round can exceed 32 bits either: the wide rounds (the first
  // ten or so of a 256-token region) hand over to the narrow ones, which run on the low words.
  // A wide round that finds the keys narrow enough returns true before it changes anything.
  unsigned long long clk[7] = {0, 0, 0, 0, 0, 0, 0};
  auto now = [&]() -> unsigned long long {
    if constexpr (CLOCKS) return __builtin_readcyclecounter(); else return 0;
  };
  auto round = [&](auto wide_c, int step) -> bool {
    constexpr bool WIDE = decltype(wide_c)::value;
    const unsigned long long t0 = now();
    using K = std::conditional_t<WIDE, uint64_t, uint32_t>;
    auto key_at = [&](int at) -> K * {
      if constexpr (WIDE) return &keys[at]; else return &keys32[at];
    };
    auto key_add = [&](int at, K by) {
      __hip_atomic_fetch_add(key_at(at), by, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto wave_max = [&](K k) -> K {
      if constexpr (WIDE) return wave_max_u64(k); else return wave_max_u32(k);
    };
    // ---- argmax of the keys (lowest index among equals) ----
    K kv[RPL], bk = 0;
    int bv = 0;
#pragma unroll
    for (int v = 0; v < RPL; v++) {
      kv[v] = *key_at(64 * v + lane);
      if (v == 0 || kv[v] > bk) { bk = kv[v]; bv = v; }
    }
    const K top = wave_max(bk);
    if constexpr (WIDE) {
      if ((top >> 32) == 0) return true;
    }
    const int tl = __builtin_ctzll(__ballot(bk == top));
    const int tv = __builtin_amdgcn_readlane(bv, tl);
    const int t = RPL * tl + tv;
    const unsigned long long t1 = now();

    // ---- the owner of column t posts row t ----
    if (w == wave_of(t)) {
      const int ct = t / NW;  // wave-uniform register index
      if constexpr (RPL == 4) {  // (the four fetches under one switch of the index mode, as in the column step below)
        int32_t q[4];
        asm volatile(
            "s_set_gpr_idx_on %[ct], gpr_idx(SRC0)\n\t"
            "v_mov_b32 %[q0], v0\n\t"
            "v_mov_b32 %[q1], v32\n\t"
            "v_mov_b32 %[q2], v64\n\t"
            "v_mov_b32 %[q3], v96\n\t"
            "s_set_gpr_idx_off"
            : [q0] "=&v"(q[0]), [q1] "=&v"(q[1]), [q2] "=&v"(q[2]), [q3] "=&v"(q[3])
            : [ct] "s"(ct), "{v[0:31]}"(sv[0]), "{v[32:63]}"(sv[1]), "{v[64:95]}"(sv[2]), "{v[96:127]}"(sv[RPL == 4 ? 3 : 0])
            : "m0");
#pragma unroll
        for (int v = 0; v < 4; v++)
          if (post_at[v] >= 0) rowt[post_at[v]] = q[v];
      } else {
#pragma unroll
        for (int v = 0; v < RPL; v++)
          if (post_at[v] >= 0) rowt[post_at[v]] = sv[v][ct];
      }
    }
    if (threadIdx.x == 0) { pick_row[step] = t; pick_val[step] = (uint64_t)top - 1u; }
    if constexpr (GAP) {
      if (w == 0) {  // the largest key among the other rows
        K sk = 0;
#pragma unroll
        for (int v = 0; v < RPL; v++) {
          const K k = (lane == tl && v == tv) ? (K)0 : kv[v];
          sk = k > sk ? k : sk;
        }
        const K second = wave_max(sk);
        if (lane == 0) pick_gap[step] = second ? (uint64_t)(top - second) : kNoRunnerUp;
      }
    }
    lds_barrier();  // every wave has read the keys; row t is posted
    const unsigned long long t2 = now();

    // ---- new coverage of the own columns; the changed ones lower the rows' values ----
    if (threadIdx.x == 0) {  // t is picked: its key ends at 0
      if constexpr (WIDE) {
        key_add(64 * tv + tl, ~(K)0);
      } else {  // (as a bare instruction: the compiler wraps an atomic on a uniform address in a count of the active lanes)
        const uint32_t at = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)&keys32[64 * tv + tl];
        asm volatile("ds_add_u32 %0, %1" ::"v"(at), "v"(~0u) : "memory");
      }
    }
    const int32_t x = rowt[32 * w + cl];
    const int32_t m_old = m;
    m = max(m, x);
    uint32_t changed = (uint32_t)__ballot(reports && x > m_old);
    const unsigned long long t3 = now();
    if constexpr (CLOCKS) clk[6] += (unsigned)__builtin_popcount(changed);
    if constexpr (!WIDE && RPL == 4) {
      // The common case (a region of 208 to 256 tokens, keys in 32-bit words) written out as
      // instructions: the column's four registers are fetched under one switch of the register-index
      // mode (instead of one switch on and off around every fetch), each bank asked for
      // in the registers where the compiler's own relative addressing keeps it anyway, and only the
      // clamped values are summed per column - the lower ends a are added up once, in a scalar
      // register (32-bit wrap-around is exact here: the true decrease fits the key's 32 bits).
      if (changed) {
        uint32_t q_sum[4] = {0u, 0u, 0u, 0u}, a_sum = 0u;
        do {
          const int c = __builtin_ctz(changed);
          changed &= changed - 1;
          const int32_t a = __builtin_amdgcn_readlane(m_old, c), b = __builtin_amdgcn_readlane(m, c);
          a_sum += (uint32_t)a;
          int32_t q0, q1, q2, q3, bv;
          asm volatile(
              "v_mov_b32 %[bv], %[b]\n\t"
              "s_set_gpr_idx_on %[c], gpr_idx(SRC0)\n\t"
              "v_mov_b32 %[q0], v0\n\t"
              "v_mov_b32 %[q1], v32\n\t"
              "v_mov_b32 %[q2], v64\n\t"
              "v_mov_b32 %[q3], v96\n\t"
              "s_set_gpr_idx_off\n\t"
              "v_med3_i32 %[q0], %[q0], %[a], %[bv]\n\t"
              "v_med3_i32 %[q1], %[q1], %[a], %[bv]\n\t"
              "v_med3_i32 %[q2], %[q2], %[a], %[bv]\n\t"
              "v_med3_i32 %[q3], %[q3], %[a], %[bv]\n\t"
              "v_add_u32 %[d0], %[d0], %[q0]\n\t"
              "v_add_u32 %[d1], %[d1], %[q1]\n\t"
              "v_add_u32 %[d2], %[d2], %[q2]\n\t"
              "v_add_u32 %[d3], %[d3], %[q3]"
              : [d0] "+v"(q_sum[0]), [d1] "+v"(q_sum[1]), [d2] "+v"(q_sum[2]), [d3] "+v"(q_sum[3]), [q0] "=&v"(q0),
                [q1] "=&v"(q1), [q2] "=&v"(q2), [q3] "=&v"(q3), [bv] "=&v"(bv)
              : [c] "s"(c), [a] "s"(a), [b] "s"(b), "{v[0:31]}"(sv[0]), "{v[32:63]}"(sv[1]), "{v[64:95]}"(sv[2]),
                "{v[96:127]}"(sv[RPL == 4 ? 3 : 0])
              : "m0");
        } while (changed);
#pragma unroll
        for (int v = 0; v < 4; v++)
          if (4 * lane + v < NL) key_add(64 * v + lane, (K)(a_sum - q_sum[v]));
      }
    } else if (changed) {
      K dec[RPL];
#pragma unroll
      for (int v = 0; v < RPL; v++) dec[v] = 0;
      do {
        const int c = __builtin_ctz(changed);
        changed &= changed - 1;
        const int32_t a = __builtin_amdgcn_readlane(m_old, c), b = __builtin_amdgcn_readlane(m, c);
#pragma unroll
        for (int v = 0; v < RPL; v++) {
          // clamp to [a, b] (a < b) as one median instruction; at most one operand may be scalar
          int32_t cl3;
          const int32_t bvec = b;
          asm("v_med3_i32 %0, %1, %2, %3" : "=v"(cl3) : "v"(sv[v][c]), "s"(a), "v"(bvec));
          dec[v] += (uint32_t)(cl3 - a);
        }
      } while (changed);
#pragma unroll
      for (int v = 0; v < RPL; v++)
        if (RPL * lane + v < NL) key_add(64 * v + lane, (K)0 - dec[v]);
    }
    const unsigned long long t4 = now();
    lds_barrier();  // the keys are final for the next round; every wave has read row t
    if constexpr (CLOCKS) {
      const unsigned long long t5 = now();
      clk[0] += t1 - t0; clk[1] += t2 - t1; clk[2] += t3 - t2; clk[3] += t4 - t3; clk[4] += t5 - t4; clk[5] += 1;
    }
    return false;
  };

  int step = 0;
  for (; step < d_loc; step++)
    if (round(std::true_type{}, step)) break;
  if (step < d_loc) {
    for (int i = threadIdx.x; i < RPL * 64; i += 64 * NW) keys32[i] = (uint32_t)keys[i];
    lds_barrier();
    for (; step < d_loc; step++) round(std::false_type{}, step);
  }
  if constexpr (CLOCKS) {
    if (lane < 8) clk_out[((size_t)bp * NW + w) * 8 + lane] = lane < 7 ? clk[lane] : 0ull;
  }
  for (int k = threadIdx.x; k < d_loc; k += 64 * NW) {
    const size_t at = (size_t)bp * d_loc + k;
    idx[at] = map.token(p, pick_row[k]);
    // the first value is the row sum shifted by N_loc (coverage -1 everywhere)
    const double val = (double)pick_val[k] - (k == 0 ? (double)NL * kSimScale : 0.0);
    if (gain_out) gain_out[at] = (float)(val / kSimScale);
    if constexpr (GAP)
      gap_out[at] = pick_gap[k] == kNoRunnerUp ? __builtin_inff() : (float)((double)pick_gap[k] / kSimScale);
  }
}

// ------------------------------------------------------------------------------------------------
// The same greedy selection for regions too large for one CU's registers (more than 256 tokens, up to
// kBigRegion: the few-regions end of the paper's region-count ablation, e.g. four regions of 1024
// tokens).  One workgroup of 1024 threads per (sample, region); S stays in global memory (it is read
// through L2), thread i owns row i and column i (and i + 1024): its row's value as a 64-bit integer and
// its column's coverage live in registers.  A round: (1) argmax of the keys - value + 1 in the high
// bits, 4095 - row in the low twelve, so the largest key is the largest value at the lowest row - by
// a wave reduction, an exchange through LDS and a second wave reduction that every wave does for
// itself; (2) every thread compares row t (one coalesced read) with its columns' coverage and appends
// the changed columns (column, old, new coverage) to a list in LDS; (3) every thread walks the list and
// lowers its rows' values by med(S_ij, m_j, m_j') - m_j, reading S_ji = S_ij along row j (coalesced).
// Integer arithmetic throughout: the values equal the full rescan of Alg. 2 whatever the order of the
// list.  Three barriers per round.
constexpr int kBigRegion = 2048, kBigThreads = 1024, kBigRows = kBigRegion / kBigThreads;

__device__ __forceinline__ uint64_t wave_max_key(uint64_t k) { return wave_max_u64(k); }

template <bool GAP>
__global__ __launch_bounds__(kBigThreads) void k_greedy_big(const int32_t *__restrict__ S, int32_t *__restrict__ idx,
                                                           float *__restrict__ gain_out, float *__restrict__ gap_out,
                                                           RegionMap map, int P, int n, int d_loc) {
  constexpr int32_t kFloor = -(1 << 30);  // similarity -1: the coverage before the first pick
  constexpr int NW = kBigThreads / 64;
  __shared__ uint64_t red[NW], red2[GAP ? NW : 1];
  __shared__ int list_n;
  __shared__ int32_t list_j[kBigRegion], list_a[kBigRegion], list_b[kBigRegion];
  const int bp = blockIdx.x, p = bp % P, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int32_t *Sr = S + (size_t)bp * n * n;

  int row[kBigRows];
  bool live[kBigRows], picked[kBigRows];
  int32_t m[kBigRows];
  uint64_t val[kBigRows];
#pragma unroll
  for (int u = 0; u < kBigRows; u++) {
    row[u] = tid + kBigThreads * u;
    live[u] = row[u] < n;
    picked[u] = false;
    m[u] = kFloor;
    val[u] = 0;
  }
  if (tid == 0) list_n = 0;
  // values under the starting coverage: sum_j (S_ij + 1), summed down the columns (S is symmetric)
  for (int j = 0; j < n; j++) {
#pragma unroll
    for (int u = 0; u < kBigRows; u++)
      if (live[u]) val[u] += (uint32_t)(Sr[(size_t)j * n + row[u]] - kFloor);
  }

  for (int step = 0; step < d_loc; step++) {
    // ---- (1) argmax ----
    uint64_t best = 0, key[kBigRows];
#pragma unroll
    for (int u = 0; u < kBigRows; u++) {
      key[u] = live[u] && !picked[u] ? ((val[u] + 1) << 12) | (uint64_t)(4095 - row[u]) : 0ull;
      best = key[u] > best ? key[u] : best;
    }
    const uint64_t wbest = wave_max_key(best);
    if (lane == 0) red[w] = wbest;
    __syncthreads();
    const uint64_t top = wave_max_key(lane < NW ? red[lane] : 0ull);
    const int t = 4095 - (int)(top & 4095);
    if constexpr (GAP) {
      uint64_t sb = 0;
#pragma unroll
      for (int u = 0; u < kBigRows; u++) {
        const uint64_t k = row[u] == t ? 0ull : key[u];
        sb = k > sb ? k : sb;
      }
      const uint64_t wsb = wave_max_key(sb);
      if (lane == 0) red2[w] = wsb;
    }
    // ---- (2) row t against the coverage of the own columns ----
#pragma unroll
    for (int u = 0; u < kBigRows; u++) {
      if (!live[u]) continue;
      const int32_t x = Sr[(size_t)t * n + row[u]];
      if (x > m[u]) {
        const int at = atomicAdd(&list_n, 1);
        list_j[at] = row[u];
        list_a[at] = m[u];
        list_b[at] = x;
        m[u] = x;
      }
      if (row[u] == t) picked[u] = true;
    }
    __syncthreads();
    if (tid == 0) {
      const size_t at = (size_t)bp * d_loc + step;
      idx[at] = map.token(p, t);
      const uint64_t value = (top >> 12) - 1;
      const double shown = (double)value - (step == 0 ? (double)n * kSimScale : 0.0);  // the first value is the row sum
      if (gain_out) gain_out[at] = (float)(shown / kSimScale);
      if constexpr (GAP) {
        uint64_t second = 0;
        for (int q = 0; q < NW; q++) second = red2[q] > second ? red2[q] : second;
        gap_out[at] = second ? (float)((double)((top >> 12) - (second >> 12)) / kSimScale) : __builtin_inff();
      }
    }
    // ---- (3) the changed columns lower the rows' values ----
    constexpr int kBatch = 4;  // list entries (rows of S) whose loads are in flight together (a round seldom has more)
    const int cnt = list_n;
    uint64_t dec[kBigRows];
#pragma unroll
    for (int u = 0; u < kBigRows; u++) dec[u] = 0;
    for (int e0 = 0; e0 < cnt; e0 += kBatch) {
      int32_t sj[kBatch][kBigRows], a[kBatch], b[kBatch];
#pragma unroll
      for (int q = 0; q < kBatch; q++) {
        const int e = min(e0 + q, cnt - 1);
        const int j = list_j[e];
        a[q] = list_a[e];
        b[q] = e0 + q < cnt ? list_b[e] : a[q];  // (a repeated entry with a == b adds nothing)
#pragma unroll
        for (int u = 0; u < kBigRows; u++) sj[q][u] = live[u] ? Sr[(size_t)j * n + row[u]] : 0;
      }
#pragma unroll
      for (int q = 0; q < kBatch; q++)
#pragma unroll
        for (int u = 0; u < kBigRows; u++) {
          const int32_t cl3 = min(max(sj[q][u], a[q]), b[q]);  // a <= b
          dec[u] += (uint32_t)(cl3 - a[q]);
        }
    }
#pragma unroll
    for (int u = 0; u < kBigRows; u++) val[u] -= dec[u];
    __syncthreads();  // everyone has read the list (and red / red2)
    if (tid == 0) list_n = 0;
  }
}

// Slices of K per 16 x 16 unit: more, smaller pieces of work spread more evenly over the SIMDs when
// the units alone are only a few per SIMD; each slice still needs a few chunks to fill its pipeline.
static int gram_k_split(const Shape &s) {
  const int tiles = s.n_loc / 16;
  const long long waves = (long long)tiles * (tiles + 1) / 2 * s.B * s.P;
  const int nchunk = s.C / 32;
  if (waves < 8 * 1024 && nchunk >= 8) return 2;
  return 1;
}

template <typename T>
static int select_typed(const Shape &s, const T *X, int32_t *idx, float *gain, float *gap, char *ws,
                        const Workspace &w, hipStream_t st, unsigned long long *parts) {
  int32_t *S = reinterpret_cast<int32_t *>(ws + w.sim);
  RegionMap map{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  const int tiles = s.n_loc / 16, units = tiles * (tiles + 1) / 2;
  RowFix fix{nullptr, nullptr, nullptr, s.N, s.C};
  if (sizeof(T) == 2 && gram_i8_workspace_bytes(s) != 0) {
    // bf16 tokens: exact similarities on the int8 matrix cores
    const double *nrm = nullptr;
    const uint8_t *flag = nullptr;
    const int rc = launch_gram_i8(s, X, S, ws + w.gram, &nrm, &flag, st);
    if (rc != TOMA_OK) return rc;
    fix = RowFix{reinterpret_cast<const bf16_t *>(X), nrm, flag, s.N, s.C};
  } else
  { KernelTimer kt(K_GRAM, st);
  if (gram_k_split(s) == 2)
    hipLaunchKernelGGL((k_gram<T, 2>), dim3((units + 1) / 2 * s.B * s.P), dim3(256), 0, st, X, S, map, s.N, s.C, s.P,
                       s.n_loc, tiles, units);
  else
    hipLaunchKernelGGL((k_gram<T, 1>), dim3((units + 3) / 4 * s.B * s.P), dim3(256), 0, st, X, S, map, s.N, s.C, s.P,
                       s.n_loc, tiles, units); }
  int regions = s.B * s.P;
  if (parts) {  // the kernel that also times the parts of its rounds (64- and 256-token regions only)
    if (s.n_loc == 256)
      hipLaunchKernelGGL((k_greedy<16, false, true>), dim3(regions), dim3(512), 0, st, S, idx, gain, nullptr, map, s.P,
                         s.d_loc, fix, parts);
    else if (s.n_loc == 64)
      hipLaunchKernelGGL((k_greedy<4, false, true>), dim3(regions), dim3(128), 0, st, S, idx, gain, nullptr, map, s.P,
                         s.d_loc, fix, parts);
    else
      return TOMA_ERR_UNSUPPORTED;
    return launch_status();
  }
  KernelTimer kt(K_GREEDY, st);
  if (s.n_loc > 256) {  // (regions too large for the register-resident kernel)
    if (gap)
      hipLaunchKernelGGL((k_greedy_big<true>), dim3(regions), dim3(kBigThreads), 0, st, S, idx, gain, gap, map, s.P, s.n_loc, s.d_loc);
    else
      hipLaunchKernelGGL((k_greedy_big<false>), dim3(regions), dim3(kBigThreads), 0, st, S, idx, gain, gap, map, s.P, s.n_loc, s.d_loc);
    return launch_status();
  }
  switch (s.n_loc / 16) {
#define TOMA_GREEDY_CASE(NT)                                                                               \
  case NT:                                                                                                 \
    if (gap)                                                                                               \
      hipLaunchKernelGGL((k_greedy<NT, true>), dim3(regions), dim3(64 * ((NT + 1) / 2)), 0, st, S, idx, gain, gap, \
                         map, s.P, s.d_loc, fix, nullptr);                                                 \
    else                                                                                                   \
      hipLaunchKernelGGL((k_greedy<NT, false>), dim3(regions), dim3(64 * ((NT + 1) / 2)), 0, st, S, idx, gain, gap, \
                         map, s.P, s.d_loc, fix, nullptr);                                                 \
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

int launch_select(const Shape &s, const void *X, int32_t *idx, float *gain, float *gap, char *ws,
                  const Workspace &w, hipStream_t st, unsigned long long *parts) {
  if (s.dtype == TOMA_BF16)
    return select_typed<bf16_t>(s, static_cast<const bf16_t *>(X), idx, gain, gap, ws, w, st, parts);
  return select_typed<float>(s, static_cast<const float *>(X), idx, gain, gap, ws, w, st, parts);
}

}  // namespace toma
