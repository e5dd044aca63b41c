// Cosine similarity of bf16 tokens on the int8 matrix cores, exactly (paper Sec. 4.1: S = cos(x_i, x_j)
// inside each region).
//
// The selection decides on similarities rounded to a grid of 2^-30 and needs them accurate far below
// that, which fp32 accumulation cannot give; the fp64 matrix cores can (k_gram) but are slow.  A bf16
// value is an 8-bit significand times a power of two, so the dot product of two tokens is an integer
// sum once every token is written in fixed point against its own largest exponent:
//     x_ic = q_ic * 2^(E_i - 156),   q_ic = +-significand << (22 - (E_i - e_ic))    (|q| < 2^30)
// and q splits into four signed bytes q = l0 + 256 l1 + 256^2 l2 + 256^3 l3 ("limbs").  Then
//     <x_i, x_j> = 2^(E_i + E_j - 312) * sum over limb pairs (a, b) of 256^(a+b) * <l_a(i), l_b(j)>,
// sixteen int8 products with int32 accumulators (exact: |sum| <= 4 * C * 2^14 < 2^31 for C <= 16384),
// added up per a + b and combined in double precision with one rounding that matters.  The int8 matrix
// cores are 64 times faster than the fp64 ones, so sixteen products still come out far ahead.
//   k_limbs    one pass over X: per token the largest exponent, the norm (double), the limb planes
//              (layout below), and for the rare element too small for the fixed point (more than 22
//              binary orders below the token's largest: about one in 10^6 elements of Gaussian data)
//              its channel and the part of its value that was dropped, which k_gram_i8's epilogue adds
//              back exactly; a token with more than a few such elements has its rows of S recomputed
//              in double precision by the selection kernel's prologue instead.
//   k_gram_i8  one workgroup per (region, 64 x 32 block of S on or above the diagonal), the two panels of
//              limbs loaded into LDS per 64 channels, 32 products per wave and chunk; the epilogue
//              scales by the tokens' norms, rounds to the grid and stores both triangles.
// Limb layout: token row = ceil(C / 64) * 64 channels; per group of 16 channels 64 bytes: limb 0 of the
// 16 channels, then limb 1, 2, 3.  A lane's operand for one limb and 16 channels is one 16-byte packet.
#include "toma_common.h"
#include "toma_gemm.h"
#include "toma_internal.h"

namespace toma {

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
constexpr int kLimbShift = 22;

// One wave per token: lane l takes the 16-channel groups l, l + 64, ... (ITER of them); the token's row
// stays in registers between finding its largest exponent and converting it, so X is read once, and
// there are as many waves as tokens to hide the memory latency of this small streaming pass.
// Elements too small for the fixed point (at most kFixMax per token are listed; more than that and the
// token's rows of S are recomputed wholesale by the selection kernel) leave a correction behind: their
// channel and the part of their value the fixed point dropped, which k_gram_i8 adds back exactly.
constexpr int kFixMax = 4;
struct LimbFix { int32_t n; int32_t ch[kFixMax]; double res[kFixMax]; };  // n > kFixMax: too many, see flag

template <int ITER>
__global__ __launch_bounds__(256) void k_limbs(const bf16_t *__restrict__ X, uint32_t *__restrict__ Xq,
                                              double *__restrict__ nrm, double *__restrict__ rnp,
                                              uint8_t *__restrict__ flag, LimbFix *__restrict__ fixes, int rows, int C,
                                              int groups_pad) {
  __shared__ int fixn[4];
  __shared__ u32x4 wbuf[4][256];  // per wave: the 256 packets of one pass over 64 groups
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, token = blockIdx.x * 4 + w;
  if (lane == 0) fixn[w] = 0;
  if (token >= rows) return;  // (whole waves leave together; nothing below crosses waves)
  const uint32_t *src = reinterpret_cast<const uint32_t *>(X + (size_t)token * C);  // two elements per word
  const int groups = C / 16;
  u32x4 pk[ITER][2];
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int g = lane + 64 * it;
    if (g < groups) {
      pk[it][0] = *reinterpret_cast<const u32x4 *>(src + 8 * g);
      pk[it][1] = *reinterpret_cast<const u32x4 *>(src + 8 * g + 4);
    } else {
      pk[it][0] = pk[it][1] = (u32x4){0u, 0u, 0u, 0u};
    }
  }
  // ---- largest exponent and sum of squares ----
  int emax = 1;
  double sq = 0.0;
#pragma unroll
  for (int it = 0; it < ITER; it++)
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const uint32_t word = pk[it][i >> 2][i & 3];
      emax = max(emax, (int)((word >> 7) & 0xffu));
      emax = max(emax, (int)((word >> 23) & 0xffu));
      const double lo = (double)__builtin_bit_cast(float, word << 16), hi = (double)__builtin_bit_cast(float, word & 0xffff0000u);
      sq = fma(lo, lo, sq);
      sq = fma(hi, hi, sq);
    }
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    emax = max(emax, __shfl_xor(emax, m, 64));
    sq += __shfl_xor(sq, m, 64);
  }
  // ---- fixed point against the largest exponent, split into limbs ----
  uint32_t *dst = Xq + (size_t)token * groups_pad * 16;
  LimbFix *fx = fixes + token;
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int g = lane + 64 * it;
    if (64 * it >= groups_pad) break;  // (uniform; lanes past the row's end carry zeros through the exchange)
    // q = trunc(x * 2^(156 - emax)): the conversion instructions do the shifting; an element that the
    // fixed point cannot hold exactly shows as a fractional part (rare: looked at once per group)
    uint32_t lq[16], inexact = 0u;
#pragma unroll
    for (int i = 0; i < 16; i++) {
      const uint32_t word = pk[it][i >> 3][(i >> 1) & 3];
      const float x = __builtin_bit_cast(float, (i & 1) ? (word & 0xffff0000u) : (word << 16));
      const float qf = __builtin_amdgcn_ldexpf(x, 156 - emax);
      inexact |= __builtin_bit_cast(uint32_t, __builtin_amdgcn_fractf(qf));
      const int32_t q = (int32_t)qf;
      // signed bytes: adding 128 to each of the three low bytes (carries and all) and flipping
      // their top bits leaves l0 + 256 l1 + 256^2 l2 + 256^3 l3 == q with every l in [-128, 127]
      lq[i] = ((uint32_t)q + 0x00808080u) ^ 0x00808080u;
    }
    if (inexact << 1) {  // (a fraction of -0 does not count)
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const uint32_t word = pk[it][i >> 3][(i >> 1) & 3];
        const uint32_t bits = (i & 1) ? (word >> 16) : (word & 0xffffu);
        const int e = (int)((bits >> 7) & 0xffu);
        const uint32_t sig = e ? (0x80u | (bits & 0x7fu)) : (bits & 0x7fu);
        const int sh = kLimbShift - (emax - max(e, 1));
        if (sh >= 0) continue;
        const int down = min(-sh, 31);
        if ((sig & ((1u << down) - 1u)) == 0u) continue;
        // what the fixed point drops: value - (+-mag) * 2^(emax - 156), exact in double
        const double val = (double)__builtin_bit_cast(float, bits << 16);
        const double kept = ldexp((double)(sig >> down), emax - 156);
        const int at = atomicAdd(&fixn[w], 1);
        if (at < kFixMax) { fx->ch[at] = 16 * g + i; fx->res[at] = val - ((bits & 0x8000u) ? -kept : kept); }
      }
    }
    // byte k of the sixteen words -> limb plane k (four words).  The four planes of a lane's group are 64
    // consecutive bytes of the token's row; they go through the wave's corner of LDS so that a store
    // instruction writes 1 KiB of consecutive bytes (lane l the packets l, l + 64, ... of this pass)
    // instead of 16-byte pieces 64 bytes apart.
    u32x4 *mine = wbuf[w];
#pragma unroll
    for (int k = 0; k < 4; k++) {
      u32x4 o;
#pragma unroll
      for (int m = 0; m < 4; m++) {
        const uint32_t sel = (uint32_t)k | ((uint32_t)(4 + k) << 8);  // byte k of the low word, byte k of the high word
        const uint32_t p01 = __builtin_amdgcn_perm(lq[4 * m + 1], lq[4 * m], sel);
        const uint32_t p23 = __builtin_amdgcn_perm(lq[4 * m + 3], lq[4 * m + 2], sel);
        o[m] = __builtin_amdgcn_perm(p23, p01, 0x05040100u);
      }
      mine[4 * lane + k] = o;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int pkt = 256 * it + 64 * j + lane;  // packet of the token's row: 4 * group + plane
      if (pkt < 4 * groups_pad) *reinterpret_cast<u32x4 *>(dst + 4 * pkt) = mine[64 * j + lane];
    }
    __builtin_amdgcn_wave_barrier();
  }
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  if (lane == 0) {
    const int nfix = __hip_atomic_load(&fixn[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    const double n = fmax(sqrt(sq), 1e-12);
    nrm[token] = n;
    rnp[token] = ldexp(1.0 / n, emax - 141);  // so that (sum of q q) * rnp_i * rnp_j = cos * 2^30
    fx->n = nfix;
    flag[token] = nfix == 0 ? 0 : (nfix <= kFixMax ? 1 : 2);  // 1: corrected by k_gram_i8; 2: recompute the rows
  }
}

// One workgroup of four waves (2 x 2) per (region, 64-token row block, 32-token column block at or right
// of the row block's diagonal): wave (wi, wj) owns the 32 x 16 block of S made of tokens 32 wi .. of the
// row block and 16 wj .. of the column block, as 2 x 1 tiles with seven int32 accumulators each (one per
// limb-index sum).  Per 64 channels the two panels (256 bytes of limbs per token) go from global memory
// straight into LDS (load-to-LDS path, no register in between: 16-byte register-to-LDS stores run at half
// the rate of the reads on this machine and were a third of the LDS's busy time) and every wave reads
// its 32 + 16 rows from there.  Units this small keep every CU of the chip busy on an SDXL-sized input
// (640 of them) and, several to a CU, hide each other's memory latency, which is what bounded 64 x 64
// units.
constexpr int kGramRow = 256;  // bytes per token and chunk in LDS: 16 packets, packet kp of row r at slot
                               // (kp & 8) | ((kp ^ r) & 7) - the swizzle of the GEMM tiles, free of bank conflicts
                               // for 16 lanes reading one packet column of 16 rows (padded rows were not)
constexpr int kGramPanel = (64 + 32) * kGramRow;  // row panel, then column panel
__device__ __forceinline__ int gram_slot(int row, int kp) { return row * kGramRow + (((kp & 8) | ((kp ^ row) & 7)) << 4); }

// with the fixed-point dot product and the norms: cos * 2^30 = dot_q * rnp_i * rnp_j.  A token whose
// fixed point dropped part of an element (flag 1) has x = xq + res on the listed channels, so
// <x_i, x_j> = <xq_i, xq_j> + sum_fix(i) res * x_j[ch] + sum_fix(j) res * xq_i[ch].
struct GramFix { const bf16_t *X; const double *nrm; const uint8_t *flag; const LimbFix *fixes; int C; };

// units of a region: row block bm (64 tokens) with the column blocks (32 tokens) 2 bm .. nb32 - 1
__host__ __device__ inline int gram_units(int n_loc) {
  const int nb64 = (n_loc + 63) / 64, nb32 = (n_loc + 31) / 32;
  int u = 0;
  for (int bm = 0; bm < nb64; bm++) u += nb32 - 2 * bm;
  return u;
}

// NBUF: LDS buffers of one chunk each - three (two workgroups per CU, two chunks in flight) when the
// grid has few workgroups per CU, two (three workgroups per CU, which hide each other's waits) otherwise
template <int NBUF>
__global__ __launch_bounds__(256, NBUF == 3 ? 2 : 3) void k_gram_i8(const uint32_t *__restrict__ Xq, const double *__restrict__ rnp,
                                                   int32_t *__restrict__ S, RegionMap map, int N, int P, int n_loc,
                                                   int row_words, int nchunks, int units, GramFix fix) {
  constexpr int kSlots = 8;  // flagged tokens of a unit that get a vector of corrections (see below)
  struct FixArea { LimbFix sfix[96]; double cvec[kSlots][64]; int8_t slot_of[96]; uint8_t flagged[kSlots]; int nflagged; };
  static_assert(sizeof(FixArea) <= NBUF * kGramPanel, "the corrections reuse the panels' memory");
  __shared__ __align__(1024) char smem[NBUF * kGramPanel];  // buffers of [64 row tokens | 32 column tokens]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const int wi = w >> 1, wj = w & 1;
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  const int bp = work / units, unit = work - bp * units;
  const int nb32 = (n_loc + 31) / 32;
  int bm = 0, rest = unit;
  while (rest >= nb32 - 2 * bm) { rest -= nb32 - 2 * bm; bm++; }
  const int bn = 2 * bm + rest;  // column block (32 tokens)
  const int b = bp / P, p = bp % P;
  const int row0 = 64 * bm, col0 = 32 * bn;

  // Staging by the load-to-LDS path: a chunk's panels are 24 KiB = 24 loads of 1 KiB, six per wave; lane l
  // of load u of wave w lands at LDS position (row 4 (6 w + u) + l / 16, slot l % 16) and therefore fetches
  // the packet that the swizzle keeps there.  Three LDS buffers: chunk k + 2 is requested while chunk k
  // is multiplied, no register holds operands in flight, and only the waits below order loads and reads.
  const uint32_t *src[6];
#pragma unroll
  for (int u = 0; u < 6; u++) {
    const int row = 4 * (6 * w + u) + (lane >> 4), slot = lane & 15;  // rows 0..63: row panel, 64..95: column panel
    const int kp = (slot & 8) | ((slot ^ row) & 7);
    const int l = min(row < 64 ? row0 + row : col0 + row - 64, n_loc - 1);
    src[u] = Xq + ((size_t)b * N + map.token(p, l)) * row_words + 4 * kp;
  }
  const uint32_t my_lds = lds_addr_of(smem) + (uint32_t)__builtin_amdgcn_readfirstlane(w) * (6 * 1024);
  auto issue = [&](int k) {  // chunk k into buffer k % 3
    const uint32_t at = my_lds + (uint32_t)(k % NBUF) * kGramPanel;
#pragma unroll
    for (int u = 0; u < 6; u++) load_to_lds16_at(src[u] + 64 * k, at + (uint32_t)u * 1024);
  };
  auto fence = [&]() { asm volatile("" ::: "memory"); };

  // does any of this unit's 96 tokens carry a correction?  (almost never; the flag is asked for here
  // and first looked at after the main loop, so its latency costs nothing)
  uint8_t my_flag = 0;
  size_t my_token = 0;
  if (tid < 96) {
    const int l = tid < 64 ? row0 + tid : col0 + tid - 64;
    my_token = (size_t)b * N + map.token(p, min(l, n_loc - 1));
    my_flag = l < n_loc ? fix.flag[my_token] : 0;
  }

  i32x4 acc[2][7];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int s = 0; s < 7; s++) acc[i][s] = (i32x4){0, 0, 0, 0};

  // this lane's operand packets: row 32 wi + 16 t + c of the row panel / 16 wj + c of the column panel,
  // channel group g, limb l
  int fa[4], fb[4];  // (rows 16 apart share their swizzle)
#pragma unroll
  for (int l = 0; l < 4; l++) {
    fa[l] = gram_slot(32 * wi + c, 4 * g + l);
    fb[l] = gram_slot(64 + 16 * wj + c, 4 * g + l);
  }
  auto products = [&](int k) {
    const char *buf = &smem[(k % NBUF) * kGramPanel];
    i32x4 a[2][4], bb[4];
#pragma unroll
    for (int l = 0; l < 4; l++) {
      bb[l] = *reinterpret_cast<const i32x4 *>(buf + fb[l]);
#pragma unroll
      for (int t = 0; t < 2; t++) a[t][l] = *reinterpret_cast<const i32x4 *>(buf + fa[l] + 16 * t * kGramRow);
    }
#pragma unroll
    for (int la = 0; la < 4; la++)
#pragma unroll
      for (int lb = 0; lb < 4; lb++)
#pragma unroll
        for (int i = 0; i < 2; i++)
          acc[i][la + lb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i][la], bb[lb], acc[i][la + lb], 0, 0, 0);
  };
  // the scaled reciprocal norms of this lane's column and eight rows: asked for now, used after the loop
  const int cl = 16 * wj + c, col = col0 + cl;
  const bool col_ok = col < n_loc;
  const size_t tj = (size_t)b * N + map.token(p, min(col, n_loc - 1));
  const double rj = rnp[tj];
  size_t ti_[2][4];
  double ri_[2][4];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      ti_[i][r] = (size_t)b * N + map.token(p, min(row0 + 32 * wi + 16 * i + 4 * g + r, n_loc - 1));
      ri_[i][r] = rnp[ti_[i][r]];
    }
  // (these loads and the flag load above have returned by the first wait: loads complete in order)
  issue(0);
  if (NBUF == 3 && nchunks > 1) issue(1);
  for (int k = 0; k < nchunks; k++) {
    // this wave's part of chunk k has landed (with three buffers chunk k + 1 may still be in flight); after
    // the barrier so has everyone's, and every wave is done with chunk k - 1, whose buffer the next request takes
    if (NBUF == 3 && k + 1 < nchunks) wait_vmcnt<6>(); else wait_vmcnt<0>();
    fence();
    __builtin_amdgcn_s_barrier();
    fence();
    if (k + NBUF - 1 < nchunks) issue(k + NBUF - 1);
    products(k);
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's reads of chunk k have returned
    fence();
  }
  __syncthreads();  // the panels are dead: their memory is used for the corrections below

  // Corrections (rare).  Slots 0..63 are the unit's row tokens, 64..95 its column tokens.  Up to kSlots
  // flagged slots get a vector of corrections each, one per partner on the other side, computed by
  // the whole workgroup with every load independent; beyond that (never seen) each element looks its
  // correction up by itself, slowly.  (The panels are dead by now: the loop ended with a barrier.)
  FixArea &fx = *reinterpret_cast<FixArea *>(smem);
  if (tid == 0) fx.nflagged = 0;
  const bool corrected = __syncthreads_or(my_flag == 1) != 0;
  bool by_element = false;
  if (corrected) {
    if (tid < 96) {
      if (my_flag == 1) {
        fx.sfix[tid] = fix.fixes[my_token];
        const int k = atomicAdd(&fx.nflagged, 1);
        fx.slot_of[tid] = (int8_t)(k < kSlots ? k : -1);
        if (k < kSlots) fx.flagged[k] = (uint8_t)tid;
      } else {
        fx.sfix[tid].n = 0;
        fx.slot_of[tid] = -1;
      }
    }
    __syncthreads();
    by_element = fx.nflagged > kSlots;
    const int nf = min(fx.nflagged, kSlots);
    for (int k = w; k < nf; k += 4) {
      // the flagged slot f and this lane's partner slot q on the other side (32 column partners only)
      const int f = fx.flagged[k];
      const bool f_is_row = f < 64;
      if (f_is_row && lane >= 32) continue;
      const int q = f_is_row ? 64 + lane : lane;
      const int lf = min(f_is_row ? row0 + f : col0 + f - 64, n_loc - 1), lq = min(f_is_row ? col0 + lane : row0 + lane, n_loc - 1);
      const size_t tf = (size_t)b * N + map.token(p, lf), tq = (size_t)b * N + map.token(p, lq);
      const LimbFix &ff = fx.sfix[f], &fq = fx.sfix[q];
      double corr = 0.0;
#pragma unroll
      for (int e = 0; e < kFixMax; e++)
        if (e < ff.n) {
          double xq = (double)(float)fix.X[tq * fix.C + ff.ch[e]];
          // a column token's dropped parts meet the row token's fixed-point value, not its full one
          if (!f_is_row)
            for (int u = 0; u < fq.n; u++)
              if (fq.ch[u] == ff.ch[e]) xq -= fq.res[u];
          corr = fma(ff.res[e], xq, corr);
        }
      fx.cvec[k][lane] = corr * 1073741824.0 / (fix.nrm[tf] * fix.nrm[tq]);
    }
    __syncthreads();
  }

  // cos * 2^30 = (sum_s acc_s 256^s) * rnp_i * rnp_j; lane holds column (token j) c and rows 4 g + r.
  // Units right of the diagonal 64 x 64 block also store the transposed element; the two units of the
  // diagonal block cover it between them.
  int32_t *Sr = S + (size_t)bp * n_loc * n_loc;
  const bool mirror = bn >= 2 * bm + 2;
#pragma unroll
  for (int i = 0; i < 2; i++) {
    i32x4 v4 = {0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int rs = 32 * wi + 16 * i + 4 * g + r, row = row0 + rs;
      if (!col_ok || row >= n_loc) continue;
      const size_t ti = ti_[i][r];
      const double ri = ri_[i][r];
      // the three high sums are exact in double (below 2^48); the low four lose at most 2^3 of 2^58 and up
      const double hi = fma((double)acc[i][6][r], 65536.0, fma((double)acc[i][5][r], 256.0, (double)acc[i][4][r]));
      const double lo = fma((double)acc[i][3][r], 16777216.0,
                            fma((double)acc[i][2][r], 65536.0, fma((double)acc[i][1][r], 256.0, (double)acc[i][0][r])));
      const double dot = fma(hi, 4294967296.0, lo);
      double cs = dot * ri * rj;
      if (corrected) {
        if (!by_element) {
          const int ki = fx.slot_of[rs], kj = fx.slot_of[64 + cl];
          if (ki >= 0) cs += fx.cvec[ki][cl];
          if (kj >= 0) cs += fx.cvec[kj][rs];
        } else {
          const LimbFix &fi = fx.sfix[rs], &fj = fx.sfix[64 + cl];
          if (fi.n | fj.n) {
            double corr = 0.0;
            for (int e = 0; e < fi.n; e++) corr = fma(fi.res[e], (double)(float)fix.X[tj * fix.C + fi.ch[e]], corr);
            for (int e = 0; e < fj.n; e++) {
              double xi = (double)(float)fix.X[ti * fix.C + fj.ch[e]];
              for (int u = 0; u < fi.n; u++)
                if (fi.ch[u] == fj.ch[e]) xi -= fi.res[u];
              corr = fma(fj.res[e], xi, corr);
            }
            cs += corr * 1073741824.0 / (fix.nrm[ti] * fix.nrm[tj]);
          }
        }
      }
      v4[r] = (int32_t)rint(cs);
      Sr[(size_t)row * n_loc + col] = v4[r];
    }
    // the transposed elements: this lane's four rows are four consecutive words of row `col`
    if (mirror && col_ok) {
      const int rb = row0 + 32 * wi + 16 * i + 4 * g;
      int32_t *mr = Sr + (size_t)col * n_loc + rb;
      if (rb + 3 < n_loc && (n_loc & 3) == 0) {
        *reinterpret_cast<i32x4 *>(mr) = v4;
      } else {
#pragma unroll
        for (int r = 0; r < 4; r++)
          if (rb + r < n_loc) mr[r] = v4[r];
      }
    }
  }
}

size_t gram_i8_workspace_bytes(const Shape &s) {
  // (channels: the limb pass keeps a token's row in registers, up to 3072 of them; work: with the limb
  // pass in front and some 10 us of fixed cost per launch (first loads, norms, double-precision
  // combination, stores) the kernel only beats the fp64 one once there is enough to do - measured in
  // 64 x 64 blocks of S times 64-channel chunks: 3200 of them win by a tenth, 7680 by a sixth, 12800 by
  // a quarter; 640 lose)
  const int nb64 = (s.n_loc + 63) / 64;
  const long long block_chunks = (long long)s.B * s.P * (nb64 * (nb64 + 1) / 2) * ((s.C + 63) / 64);
  // (regions of more than 256 tokens take the selection kernel that has no fallback for flagged tokens)
  if (s.dtype != TOMA_BF16 || s.C > 3072 || block_chunks < 3000 || s.n_loc > 256) return 0;
  const size_t rows = (size_t)s.B * s.N;
  const size_t words = (size_t)((s.C + 63) / 64) * 64;  // one word (four limbs) per channel of the padded row
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  return up(rows * words * 4) + 2 * up(rows * sizeof(double)) + up(rows) + up(rows * sizeof(LimbFix));
}

// S for every region of a bf16 input; ws_part: gram_i8_workspace_bytes() bytes.  Leaves the per-token
// norms and flags where the selection kernel's prologue finds them (returned through the pointers).
int launch_gram_i8(const Shape &s, const void *X, int32_t *S, char *ws_part, const double **nrm_out,
                   const uint8_t **flag_out, hipStream_t st) {
  const size_t rows = (size_t)s.B * s.N;
  const int nchunks = (s.C + 63) / 64, row_words = nchunks * 64, groups_pad = nchunks * 4;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  uint32_t *Xq = reinterpret_cast<uint32_t *>(ws_part);
  double *nrm = reinterpret_cast<double *>(ws_part + up(rows * row_words * 4));
  double *rnp = reinterpret_cast<double *>(reinterpret_cast<char *>(nrm) + up(rows * sizeof(double)));
  uint8_t *flag = reinterpret_cast<uint8_t *>(reinterpret_cast<char *>(rnp) + up(rows * sizeof(double)));
  LimbFix *fixes = reinterpret_cast<LimbFix *>(reinterpret_cast<char *>(flag) + up(rows));
  RegionMap map{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  {
    KernelTimer kt(K_LIMBS, st);
    const dim3 grid((unsigned)((rows + 3) / 4));
    const bf16_t *Xb = static_cast<const bf16_t *>(X);
    const int iter = (groups_pad + 63) / 64;  // (the padded row: its zero groups are written too)
#define TOMA_LIMBS_CASE(IT) \
  hipLaunchKernelGGL(k_limbs<IT>, grid, dim3(256), 0, st, Xb, Xq, nrm, rnp, flag, fixes, (int)rows, s.C, groups_pad)
    if (iter <= 1) TOMA_LIMBS_CASE(1);
    else if (iter <= 2) TOMA_LIMBS_CASE(2);
    else if (iter <= 3) TOMA_LIMBS_CASE(3);
    else return TOMA_ERR_UNSUPPORTED;
#undef TOMA_LIMBS_CASE
  }
  const int units = gram_units(s.n_loc), regions = s.B * s.P;
  KernelTimer kt(K_GRAM, st);
  const GramFix gfix{static_cast<const bf16_t *>(X), nrm, flag, fixes, s.C};
  if ((long long)units * regions <= 2 * 256)
    hipLaunchKernelGGL(k_gram_i8<3>, dim3(units * regions), dim3(256), 0, st, Xq, rnp, S, map, s.N, s.P, s.n_loc, row_words,
                       nchunks, units, gfix);
  else
    hipLaunchKernelGGL(k_gram_i8<2>, dim3(units * regions), dim3(256), 0, st, Xq, rnp, S, map, s.N, s.P, s.n_loc, row_words,
                       nchunks, units, gfix);
  *nrm_out = nrm;
  *flag_out = flag;
  return launch_status();
}

}  // namespace toma
