// Merge weights, merge and transpose unmerge (paper Sec. 4.2.1, Sec. 4.2.2; Alg. 3 steps 2-3).
//
// Weights.  Inside a merge region the logits L[s][j] = scale * <x_s, x_idx[j]> form a
// (sources x destinations) product; the softmax runs over destinations j for each source s
// ("column-wise" in the paper's D x N orientation).  Two passes over the same MFMA product:
//   pass 1  per source row: max and sum of exp over each 64-destination slice of the tile,
//           combined by k_lse into lse[s] = max + log(sum);
//   pass 2  recompute the logits, A[j][s] = exp(L - lse[s]) stored destination-major in dtype, and
//           partial row sums of the STORED values, combined in a fixed order by k_zsum into Z[j].
// The logits stay in fp32 until after the max-subtracted exponential (at tau = 0.1 and width 640
// they reach several thousand, far beyond what bf16 could resolve).
// Merge.    Xm = diag(1/Z) A X: A is the k-contiguous left operand, X the k-major right operand.
// Unmerge.  Y = A^T diag(1/Z) O: both operands are k-major; O is scaled by 1/Z beforehand.
// The destination gather X[idx] and the region split / reassembly are address arithmetic inside
// the tile loads and stores; no token is ever copied into a region-major layout.
#include <type_traits>

#include "toma_gemm.h"
#include "toma_internal.h"
#include "toma_region.h"

namespace toma {

// ---- pass 1 and pass 2 of the weights ----------------------------------------------------------
template <typename T, bool WRITE> struct WeightsPol {
  static constexpr bool A_KS = false, B_KS = false, SPLIT_K = false, ACC_T = false;
  static constexpr int EPI = 3;
  static constexpr bool EPI_LDS = WRITE;
  RegionView<T> v;
  const int32_t *idx;
  float scale;
  float2 *stats;   // pass 1 out: [B*R][Nr][parts]
  int parts;
  const float *lse;  // pass 2 in: [B*R][Nr]
  T *A;              // pass 2 out: [B*R][Dr][lda], lda >= Nr
  int lda;
  float *zpart;      // pass 2 out: [B*R][Dr][zparts] (null: not wanted)
  int zparts;
  uint8_t *occ;      // pass 2 out (optional): occupancy map of A, zeroed before the launch
  int occ_db, occ_sb;
  // Pass 2 may skip the product of a tile that pass 1's statistics prove empty: pass 1 left, per
  // source row and slice of `slice` destinations, the largest logit of the slice; where every such
  // maximum of a tile lies more than kEmptyGap below its row's log-sum-exp, every weight of the tile
  // is below exp(-kEmptyGap), which rounds to zero in bf16 and in fp32 alike, and the tile is
  // written as zeros.  (With a small temperature that is all but the tiles around a token's own
  // region.)
  static constexpr bool EMPTY_TILES = WRITE;
  static constexpr float kEmptyGap = 110.0f;
  const float2 *seen;  // pass 1's statistics (null: no skipping)
  int seen_parts, slice;
  __device__ __forceinline__ bool tile_is_empty(const GemmCtx &x, int m0, int n0, int bm, int bn, int tid,
                                                int nthreads) const {
    if (!WRITE || !seen) return false;
    const int p0 = n0 / slice, p1 = min((min(n0 + bn, x.N) - 1) / slice, seen_parts - 1);
    for (int t = tid; t < bm; t += nthreads) {
      const int m = m0 + t;
      if (m >= x.M) break;
      const float l = lse[(size_t)x.z * x.M + m];
      const float2 *row = seen + ((size_t)x.z * x.M + m) * seen_parts;
      for (int q = p0; q <= p1; q++)
        if (!(row[q].x - l < -kEmptyGap)) return false;
    }
    return true;
  }
  __device__ __forceinline__ void write_empty_tile(const GemmCtx &x, int m0, int n0, int bm, int bn, int wave_rows,
                                                   int tid, int nthreads) const {
    constexpr int EPC = 16 / (int)sizeof(T);
    const int m1 = min(m0 + bm, x.M), n1 = min(n0 + bn, x.N);
    const int cpr = (m1 - m0) / EPC;  // 16-byte chunks per destination row (M is a multiple of 16)
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int e = tid; e < (n1 - n0) * cpr; e += nthreads) {
      const int n = n0 + e / cpr, m = m0 + (e % cpr) * EPC;
      *reinterpret_cast<u32x4 *>(A + ((size_t)x.z * x.N + n) * lda + m) = zero;
    }
    // the partial row sums of all of this tile's wave slices (also those past a ragged end: the
    // row-sum kernel adds up every slice of every tile)
    if (!zpart) return;  // (the merge product makes Z)
    const int parts = bm / wave_rows, part0 = m0 / wave_rows;
    for (int e = tid; e < (n1 - n0) * parts; e += nthreads)
      zpart[((size_t)x.z * x.N + n0 + e / parts) * zparts + part0 + e % parts] = 0.f;
  }
  __device__ __forceinline__ GemmCtx setup(int bz) const {
    return GemmCtx{v.Nr, v.Dr, v.C, bz / v.R, bz % v.R, bz};
  }
  __device__ __forceinline__ bool a_linear(int) const { return true; }
  __device__ __forceinline__ bool b_linear(int) const { return true; }
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &x, int m, int k) const {
    return v.X + ((size_t)x.b * v.N + v.token(x.rho, m)) * v.C + k;
  }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &x, int n, int k) const {
    int t = idx[(size_t)x.b * v.D + x.rho * v.Dr + n];
    t = t < 0 ? 0 : (t >= v.N ? v.N - 1 : t);
    return v.X + ((size_t)x.b * v.N + t) * v.C + k;
  }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane, void *wave_lds) const {
    const int g = lane >> 4, c = lane & 15;
    const int M = x.M, N = x.N, z = x.z;
    if (!WRITE) {
      // per source row: (max, sum exp) over this wave's slice of destination columns
      const int part = n_w / (16 * TN);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
          float mx = -__builtin_inff();
#pragma unroll
          for (int j = 0; j < TN; j++) {
            int n = n_w + 16 * j + c;
            if (n < N) mx = fmaxf(mx, acc.t[i][j][r] * scale);
          }
          mx = row16_max_f32(mx);
          float sum = 0.f;
#pragma unroll
          for (int j = 0; j < TN; j++) {
            int n = n_w + 16 * j + c;
            if (n < N) sum += __expf(acc.t[i][j][r] * scale - mx);
          }
          sum = row16_sum_f32(sum);
          int m = m_w + 16 * i + 4 * g + r;
          if (c == 0 && m < M) stats[((size_t)z * M + m) * parts + part] = make_float2(mx, sum);
        }
    } else {
      float colsum[TN];
#pragma unroll
      for (int j = 0; j < TN; j++) colsum[j] = 0.f;
      // occupancy: a wave's tile lies inside one block of destinations and covers one or two
      // blocks of sources
      constexpr int kSrcBlocks = 16 * TM > kOccSrc ? 16 * TM / kOccSrc : 1;
      bool nonzero[kSrcBlocks];
#pragma unroll
      for (int h = 0; h < kSrcBlocks; h++) nonzero[h] = false;
#pragma unroll
      for (int i = 0; i < TM; i++) {
        int mb = m_w + 16 * i + 4 * g;  // four consecutive sources mb .. mb+3 (M is a multiple of 16)
        if (mb >= M) continue;
        float l4[4];
#pragma unroll
        for (int r = 0; r < 4; r++) l4[r] = lse[(size_t)z * M + mb + r];
#pragma unroll
        for (int j = 0; j < TN; j++) {
          int n = n_w + 16 * j + c;
          if (n >= N) continue;
          alignas(16) T o[4];
#pragma unroll
          for (int r = 0; r < 4; r++) {
            o[r] = from_f32<T>(__expf(acc.t[i][j][r] * scale - l4[r]));
            const float stored = to_f32(o[r]);
            colsum[j] += stored;
            nonzero[16 * i / kOccSrc % kSrcBlocks] |= stored != 0.f;
          }
          // straight to memory (8 / 16 bytes per lane), or into this wave's LDS scratch: row = the
          // destination, 16-byte chunk u of a row at position u ^ (row & 7)
          T *dst;
          if (wave_lds) {
            constexpr int EPC = 16 / (int)sizeof(T);  // elements per chunk
            const int nl = 16 * j + c, ml = 16 * i + 4 * g;
            constexpr int CPR = 16 * TM / EPC;        // chunks per row (a power of two)
            dst = static_cast<T *>(wave_lds) + nl * (16 * TM) + (((ml / EPC) ^ (nl & (CPR - 1) & 7)) * EPC) + ml % EPC;
          } else {
            dst = A + ((size_t)z * N + n) * lda + mb;
          }
          if (sizeof(T) == 2) {
            *reinterpret_cast<u32x2 *>(dst) = *reinterpret_cast<u32x2 *>(o);
          } else {
            *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<u32x4 *>(o);
          }
        }
      }
      if (wave_lds) {
        // whole destination rows of the wave tile (16 TM sources = 128 / 256 bytes) leave as 16-byte
        // packets of consecutive lanes: full cache lines instead of 32-byte pieces
        constexpr int EPC = 16 / (int)sizeof(T), CPR = 16 * TM / EPC;  // chunks per row
        constexpr int RPP = 64 / CPR;                                   // rows per pass
        const int u = lane % CPR, rl = lane / CPR;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // LDS is in order within the wave; this pins the compiler
#pragma unroll
        for (int p = 0; p < 16 * TN / RPP; p++) {
          const int nl = p * RPP + rl, n = n_w + nl, m = m_w + u * EPC;
          const u32x4 pk = *reinterpret_cast<const u32x4 *>(static_cast<const T *>(wave_lds) + nl * (16 * TM) +
                                                             ((u ^ (nl & (CPR - 1) & 7)) * EPC));
          if (n < N && m < M) *reinterpret_cast<u32x4 *>(A + ((size_t)z * N + n) * lda + m) = pk;
        }
      }
      if (occ) {
        // every wave that found a nonzero value stores a one (the map starts at zero; several
        // waves may store the same one)
#pragma unroll
        for (int h = 0; h < kSrcBlocks; h++) {
          const int sblk = m_w / kOccSrc + h, dblk = n_w / kOccDest;
          if (__any(nonzero[h]) && lane == 0 && sblk < occ_sb && dblk < occ_db)
            occ[((size_t)z * occ_db + dblk) * occ_sb + sblk] = 1;
        }
      }
      const int part = m_w / (16 * TM);
      if (zpart) {
#pragma unroll
        for (int j = 0; j < TN; j++) {
          float v4 = colsum[j];
          v4 += wave_xor_f32(v4, 16);
          v4 += wave_xor_f32(v4, 32);
          int n = n_w + 16 * j + c;
          if (g == 0 && n < N) zpart[((size_t)z * N + n) * zparts + part] = v4;
        }
      }
    }
  }
};

// lse[row] = M + log(sum_i s_i exp(m_i - M)) over the row's partial (max, sum) pairs.  One 16-lane
// group per row, partials strided over its lanes; the combination order is fixed.
// On the side it zeroes `zero_words` 32-bit words at `zero` (the occupancy map the write pass that
// follows fills with ones), so that this needs no launch of its own.
// (lse2, optional: the same as the pair (M, log sum), which keeps the bits that M + log sum rounds away)
__global__ __launch_bounds__(256) void k_lse(const float2 *__restrict__ stats, float *__restrict__ lse,
                                            float2 *__restrict__ lse2, int rows, int stride, int parts,
                                            uint32_t *__restrict__ zero, size_t zero_words) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < zero_words; i += (size_t)gridDim.x * 256) zero[i] = 0;
  int row = (blockIdx.x * 256 + threadIdx.x) >> 4, c = threadIdx.x & 15;
  if (row >= rows) return;
  const float2 *s = stats + (size_t)row * stride;
  float mx = -__builtin_inff();
  for (int i = c; i < parts; i += 16) mx = fmaxf(mx, s[i].x);
  mx = row16_max_f32(mx);
  float sum = 0.f;
  for (int i = c; i < parts; i += 16) sum += s[i].y * __expf(s[i].x - mx);
  sum = row16_sum_f32(sum);
  if (c == 0) {
    const float ls = __logf(sum);
    lse[row] = mx + ls;
    if (lse2) lse2[row] = make_float2(mx, ls);
  }
}

// Z[j] = sum of the partial row sums (fixed order: reruns are bit-identical).
__global__ __launch_bounds__(256) void k_zsum(const float *__restrict__ zpart, float *__restrict__ Z, int rows,
                                             int stride, int parts) {
  int row = (blockIdx.x * 256 + threadIdx.x) >> 4, c = threadIdx.x & 15;
  if (row >= rows) return;
  const float *s = zpart + (size_t)row * stride;
  float sum = 0.f;
  for (int i = c; i < parts; i += 16) sum += s[i];
  sum = row16_sum_f32(sum);
  if (c == 0) Z[row] = sum;
}

// The softmax over destinations and the stores of the one-pass kernel below.  acc[i][j] holds the
// raw products of source rows 16 i + 4 g + r against destination 16 NJ w + 16 j + c; red / rowstat are
// the workgroup's exchange buffers.
template <typename T, int NJ>
__device__ __forceinline__ void weights_one_pass_finish(f32x4 (&acc)[2][NJ], const RegionView<T> &v, float scale,
                                                        T *__restrict__ A, int lda, float *__restrict__ zpart, int zparts,
                                                        uint8_t *__restrict__ occ, int occ_db, int occ_sb,
                                                        float (&red)[8][32], float (&rowstat)[32], int z, int mt) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const int m0 = 32 * mt;
  // ---- softmax over the destinations of every source row ----
  // lane holds, of rows 16 i + 4 g + r, the columns 16 j + c of its wave's slice.  One exponential
  // per value: e = 2^((acc - max) scale log2 e) replaces acc, and the stored weight is e / sum(e).
  // (scale > 0, so the largest raw product is the largest logit; the fused multiply-add rounds
  // (acc - max) scale once, which keeps the exponent of a logit of several thousand to ~1e-6)
  const float k2 = scale * 1.44269504088896341f;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      float m = -__builtin_inff();
#pragma unroll
      for (int j = 0; j < NJ; j++) m = fmaxf(m, acc[i][j][r]);
      m = row16_max_f32(m);
      if (c == 0) red[w][16 * i + 4 * g + r] = m;
    }
  __syncthreads();
  if (tid < 32) {
    float m = red[0][tid];
#pragma unroll
    for (int ww = 1; ww < 8; ww++) m = fmaxf(m, red[ww][tid]);
    rowstat[tid] = m;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const float mk = rowstat[16 * i + 4 * g + r] * k2;
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        acc[i][j][r] = __builtin_amdgcn_exp2f(fmaf(acc[i][j][r], k2, -mk));
        sum += acc[i][j][r];
      }
      sum = row16_sum_f32(sum);
      if (c == 0) red[w][16 * i + 4 * g + r] = sum;  // (every wave read rowstat after the barrier above)
    }
  __syncthreads();
  if (tid < 32) {
    float sum = red[0][tid];
#pragma unroll
    for (int ww = 1; ww < 8; ww++) sum += red[ww][tid];  // fixed order
    rowstat[tid] = 1.0f / sum;                           // (the row's largest logit contributes 1: sum >= 1)
  }
  __syncthreads();
  // ---- A[j][s] = exp(L - lse[s]) = e / sum in dtype, destination-major; partial row sums of the stored values ----
  float l4[2][4];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) l4[i][r] = rowstat[16 * i + 4 * g + r];
  // occupancy of this wave's block(s) of A (kOccDest destinations x the workgroup's kOccSrc sources):
  // any stored value that is not zero?  (occ is only passed when a wave's slice is whole blocks)
  constexpr int kBlocks = 16 * NJ >= kOccDest ? 16 * NJ / kOccDest : 1;
  bool nonzero[kBlocks];
#pragma unroll
  for (int h = 0; h < kBlocks; h++) nonzero[h] = false;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int n = w * 16 * NJ + 16 * j + c;
    float colsum = 0.f;
    alignas(16) T o[2][4];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        o[i][r] = from_f32<T>(acc[i][j][r] * l4[i][r]);
        const float stored = to_f32(o[i][r]);
        colsum += stored;
        nonzero[16 * j / kOccDest % kBlocks] |= stored != 0.f;
      }
    T *row = A + ((size_t)z * v.Dr + n) * lda + m0;
    if constexpr (sizeof(T) == 2) {
      // A lane holds 8 bytes of each source tile (four sources); lanes g and g ^ 1 trade halves so
      // that each stores one 16-byte packet and the four lanes of a destination a whole 64-byte run
      // (even g: sources 4 g .. 4 g + 7 of tile 0, odd g: sources 4 (g - 1) .. 4 g + 3 of tile 1)
      const u32x2 own0 = *reinterpret_cast<u32x2 *>(o[0]), own1 = *reinterpret_cast<u32x2 *>(o[1]);
      const bool odd = g & 1;
      const u32x2 give = odd ? own0 : own1;
      u32x2 got;
      got[0] = (uint32_t)__shfl_xor((int)give[0], 16, 64);
      got[1] = (uint32_t)__shfl_xor((int)give[1], 16, 64);
      const u32x4 pk = odd ? (u32x4){got[0], got[1], own1[0], own1[1]} : (u32x4){own0[0], own0[1], got[0], got[1]};
      *reinterpret_cast<u32x4 *>(row + (odd ? 16 + 4 * (g - 1) : 4 * g)) = pk;
    } else {
#pragma unroll
      for (int i = 0; i < 2; i++) *reinterpret_cast<u32x4 *>(row + 16 * i + 4 * g) = *reinterpret_cast<u32x4 *>(o[i]);
    }
    if (zpart) {  // (null: the merge product that follows makes Z from its own A fragments)
      colsum += wave_xor_f32(colsum, 16);
      colsum += wave_xor_f32(colsum, 32);
      if (g == 0) zpart[((size_t)z * v.Dr + n) * zparts + mt] = colsum;
    }
  }
  if (occ) {
    static_assert(kOccSrc == 32, "one source block per workgroup");
#pragma unroll
    for (int h = 0; h < kBlocks; h++) {
      const bool any = __any(nonzero[h]);
      if (lane == 0) occ[((size_t)z * occ_db + w * kBlocks + h) * occ_sb + mt] = any ? 1 : 0;
    }
  }
}

// ---- weights in one pass ------------------------------------------------------------------------
// One workgroup (8 waves) holds the logits of 32 sources against ALL Dr = 128 NJ destinations of the
// merge region in its accumulators (wave w: destinations 16 NJ w .. 16 NJ (w + 1) - 1, 2 x NJ MFMA
// tiles), so the softmax over destinations needs no second product: the statistics are exchanged
// through LDS and A is written straight from the accumulators.
// A K step is 128 bytes of every row: two 32-channel fragments (bf16) or one (fp32).  A destination
// row is used by one wave only: every wave streams its own rows through a PRIVATE ring of LDS
// stages (two MFMA tiles = 4 KiB each) with the load-to-LDS path, three stages ahead of the
// products, and only its own s_waitcnt orders them.  The 32 source rows of a step are shared: four
// waves fetch them into a double buffer and the workgroup meets once per K step.
// Partial row sums of the STORED weights go to zpart[.][source tile] for k_zsum, as in the
// two-pass path.
template <typename T, int NJ>
__global__ __launch_bounds__(512) void k_weights_fused(const RegionView<T> v, const int32_t *__restrict__ idx, float scale,
                                                     T *__restrict__ A, int lda, float *__restrict__ zpart,
                                                     int zparts, uint8_t *__restrict__ occ, int occ_db, int occ_sb,
                                                     int tiles) {
  constexpr int ES = (int)sizeof(T), EPS = 128 / ES;   // elements per K step
  constexpr int EPP = 16 / ES;
  constexpr int NH = ES == 2 ? 2 : 1;                  // fragments per row per K step
  constexpr int JS = NJ < 2 ? 1 : 2;                   // MFMA tiles per stage
  constexpr int SPS = NJ / JS;                         // stages per K step
  constexpr int RS = 4;                                // ring stages per wave
  constexpr int LPS = 2 * JS;                          // load instructions (1 KiB) per stage
  constexpr int STAGE = JS * 16 * EPS;                 // elements per stage
  __shared__ __align__(1024) T Bs[8][RS][2 * 16 * EPS];  // per wave ring (sized for two tiles per stage)
  __shared__ __align__(1024) T As[2][32 * EPS];          // the step's 32 source rows, double buffered
  __shared__ float red[8][32];       // per wave partial statistic of the 32 source rows
  __shared__ float rowstat[32];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  // Every workgroup of a region streams the region's whole set of destination rows: the workgroups an
  // XCD receives are consecutive source tiles of as few regions as possible, so that those rows stay
  // in its L2 (two samples' rows at SDXL's first stage would not fit one L2 together).
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  const int z = work / tiles, mt = work - z * tiles, b = z / v.R, rho = z % v.R;
  const int m0 = mt * 32;
  const T *Xb = v.X + (size_t)b * v.N * v.C;

  // what this lane fetches of a 1 KiB chunk (8 rows x 128 bytes): row lane / 8, and the packet that
  // the swizzle places at position lane % 8 of that row
  const int l_row = lane >> 3;
  const int l_pkt = ((lane & 7) ^ (l_row & 7)) * EPP;
  // Element offsets (inside the sample) of the packets this lane fetches of its wave's destination
  // rows, one per (stage of a K step, chunk): the same for every K step, so they stay in registers.
  int roff[SPS][LPS];
#pragma unroll
  for (int q = 0; q < SPS; q++)
#pragma unroll
    for (int ch = 0; ch < LPS; ch++) {
      int t = idx[(size_t)b * v.D + rho * v.Dr + w * 16 * NJ + 16 * (q * JS + (ch >> 1)) + 8 * (ch & 1) + l_row];
      t = t < 0 ? 0 : (t >= v.N ? v.N - 1 : t);
      roff[q][ch] = t * v.C + l_pkt;
    }
  // source rows: wave w < 4 fetches rows 8 w .. 8 w + 7 of every step
  const T *a_src = Xb + (size_t)v.token(rho, m0 + 8 * (w & 3) + l_row) * v.C + l_pkt;
  const int nsteps = v.C / EPS, U = nsteps * SPS;
  // LDS byte addresses (scalar registers) of this wave's ring and of its part of the source rows
  const uint32_t w_s = (uint32_t)__builtin_amdgcn_readfirstlane(w);
  const uint32_t bs_lds = lds_addr_of(&Bs[0][0][0]) + w_s * (RS * 2 * 16 * EPS * ES);
  const uint32_t as_lds = lds_addr_of(&As[0][0]) + (w_s & 3) * 1024;
  auto issue_a = [&](int s) { load_to_lds16_at(a_src + s * EPS, as_lds + (uint32_t)(s & 1) * (32 * EPS * ES)); };
  // stage u = s * SPS + q of the ring (q is a compile-time constant at every call)
  auto issue_b = [&](int s, int q) {
    const uint32_t dst = bs_lds + (uint32_t)((s * SPS + q) & (RS - 1)) * (2 * 16 * EPS * ES);
    const T *src = Xb + s * EPS;
#pragma unroll
    for (int ch = 0; ch < LPS; ch++) load_to_lds16_at(src + roff[q][ch], dst + ch * 1024);
  };
  auto fence = [&]() { asm volatile("" ::: "memory"); };

  f32x4 acc[2][NJ];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < NJ; j++) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // the index loads above have returned (their values were used): from here on vmcnt counts
  // only ring loads
  wait_vmcnt<0>();
  if (w < 4) issue_a(0);
#pragma unroll
  for (int u = 0; u < RS - 1; u++)
    if (u < U) issue_b(u / SPS, u % SPS);
  wait_vmcnt<0>();
  fence();
  __builtin_amdgcn_s_barrier();
  fence();

  for (int s = 0; s < nsteps; s++) {
    if (w < 4 && s + 1 < nsteps) issue_a(s + 1);
    Frag<T> fa[2][NH];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int h = 0; h < NH; h++) frag_load_kc_sw(fa[i][h], As[s & 1], 16 * i + c, 32 * h + 8 * g);
#pragma unroll
    for (int q = 0; q < SPS; q++) {
      const int u = s * SPS + q;
      if (u + RS - 1 < U) issue_b(s + (q + RS - 1) / SPS, (q + RS - 1) % SPS);
      // this wave's loads of stage u are the oldest outstanding ones
      const int younger = min(U - 1 - u, RS - 1);
      if (younger >= 3) wait_vmcnt<3 * LPS>();
      else if (younger == 2) wait_vmcnt<2 * LPS>();
      else if (younger == 1) wait_vmcnt<LPS>();
      else wait_vmcnt<0>();
      fence();
      const T *bt = Bs[w][u & (RS - 1)];
#pragma unroll
      for (int t = 0; t < JS; t++)
#pragma unroll
        for (int h = 0; h < NH; h++) {
          Frag<T> fb;
          frag_load_kc_sw(fb, bt, 16 * t + c, 32 * h + 8 * g);
#pragma unroll
          for (int i = 0; i < 2; i++) mma16(acc[i][q * JS + t], fa[i][h], fb);
        }
      // the fragment reads of this stage have returned before its slot is refilled (next trip)
      __builtin_amdgcn_s_waitcnt(0xc07f);
      fence();
    }
    // the next step's source rows have landed (they are older than the ring loads issued during a
    // long step; a short step waits for them explicitly), and every wave is done with this step's
    constexpr int kAfterA = SPS * LPS < (RS - 1) * LPS ? SPS * LPS : (RS - 1) * LPS;
    if ((s + 1) * SPS + RS - 1 <= U) wait_vmcnt<kAfterA>();  // every stage of this step issued a refill after them
    else wait_vmcnt<0>();                                     // (the last steps issue fewer)
    fence();
    __builtin_amdgcn_s_barrier();
    fence();
  }

  weights_one_pass_finish<T, NJ>(acc, v, scale, A, lda, zpart, zparts, occ, occ_db, occ_sb, red, rowstat, z, mt);
}

// ---- merge -------------------------------------------------------------------------------------
// Occupancy map of A as the two products read it: [region][destination block][source block] bytes.
struct OccMap {
  const uint8_t *map;  // null: every block counts as occupied
  int db, sb;          // blocks per region
  // any nonzero block among destinations [j0, j1) x sources [k0, k1) of region z?
  __device__ __forceinline__ bool any(int z, int j0, int j1, int k0, int k1) const {
    const int d0 = j0 / kOccDest, d1 = min((j1 - 1) / kOccDest, db - 1);
    const int s0 = k0 / kOccSrc, s1 = min((k1 - 1) / kOccSrc, sb - 1);
    const uint8_t *row = map + ((size_t)z * db + d0) * sb;
    uint32_t acc = 0;
    for (int d = d0; d <= d1; d++, row += sb)
      for (int q = s0; q <= s1; q++) acc |= row[q];
    return acc != 0;
  }
};

template <typename T> struct MergePol {
  static constexpr bool A_KS = false, B_KS = true, SPLIT_K = true, ACC_T = true, SPARSE_K = true, ROW_SUMS = true;
  static constexpr int EPI = 1;
  static constexpr bool EPI_LDS = false;
  OccMap occ;
  __host__ __device__ __forceinline__ bool k_list() const { return occ.map != nullptr; }
  // K runs over the sources, M over the destinations
  __device__ __forceinline__ bool k_active(const GemmCtx &x, int m0, int bm, int k0, int bk) const {
    return occ.any(x.z, m0, min(m0 + bm, x.M), k0, min(k0 + bk, x.K));
  }
  RegionView<T> v;
  const T *A;  // [B*R][Dr][lda]
  int lda;
  const float *Z;
  // Z made here instead (null: read Z): the row sums of A fall out of the product's own A fragments, so
  // fresh weights need no reduction kernel of their own.  Only with K whole in every workgroup.
  float *Zout;
  __host__ __device__ __forceinline__ bool row_sums() const { return Zout != nullptr; }
  T *Xm;
  float *part;
  __device__ __forceinline__ float *split_buffer() const { return part; }
  __device__ __forceinline__ void finish(const GemmCtx &x, int m, int n, f32x4 acc) const {
    const size_t row = (size_t)x.b * v.D + x.rho * v.Dr + m;
    store4<T>(Xm + row * v.C + n, acc * (1.0f / fmaxf(Z[row], 1e-20f)));
  }
  __device__ __forceinline__ GemmCtx setup(int bz) const {
    return GemmCtx{v.Dr, v.C, v.Nr, bz / v.R, bz % v.R, bz};
  }
  __device__ __forceinline__ bool a_linear(int) const { return true; }
  __device__ __forceinline__ bool b_linear(int step) const { return v.token_linear(step); }
  // where B is not linear in k it may still move as a whole from step to step: every packet of the
  // step starting at source k sits b_step_offset(k) elements past its place in the step at source 0
  static constexpr bool B_STEP_OFFSET = true;
  __device__ __forceinline__ bool b_step_uniform(int step) const { return v.token_step_uniform(step); }
  __device__ __forceinline__ ptrdiff_t b_step_offset(const GemmCtx &x, int k) const {
    return (ptrdiff_t)(v.token(x.rho, k) - v.token(x.rho, 0)) * v.C;
  }
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &x, int m, int k) const {
    return A + ((size_t)x.z * x.M + m) * lda + k;
  }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &x, int n, int k) const {
    return v.X + ((size_t)x.b * v.N + v.token(x.rho, k)) * v.C + n;
  }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane, void *wave_lds) const {
    const float *Zr = Z + (size_t)x.b * v.D + x.rho * v.Dr;
    T *out = Xm + ((size_t)x.b * v.D + x.rho * v.Dr) * v.C;
    const int Cc = v.C;
    if (Zout) {
      // lane holds row m = m_w + 16 i + c (four consecutive columns of it per tile) and that row's sum
      const int g = lane >> 4, c = lane & 15;
      float *Zw = Zout + (size_t)x.b * v.D + x.rho * v.Dr;
#pragma unroll
      for (int i = 0; i < TM; i++) {
        const int m = m_w + 16 * i + c;
        if (m >= x.M) continue;
        const float zsum = acc.rs[i][0];
        if (n_w == 0 && g == 0) Zw[m] = zsum;
        const float sc = 1.0f / fmaxf(zsum, 1e-20f);
#pragma unroll
        for (int j = 0; j < TN; j++) {
          const int n = n_w + 16 * j + 4 * g;
          if (n < x.N) store4<T>(out + (size_t)m * Cc + n, acc.t[i][j] * sc);
        }
      }
      return;
    }
    store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N,
                  [=](int m) { return out + (size_t)m * Cc; }, [](int n) { return n; },
                  [=](int m) { return 1.0f / fmaxf(Zr[m], 1e-20f); });
  }
};

// ---- unmerge -----------------------------------------------------------------------------------
template <typename T> struct UnmergePol {
  static constexpr bool A_KS = true, B_KS = true, SPLIT_K = true, ACC_T = true, SPARSE_K = true;
  static constexpr int EPI = 1;
  static constexpr bool EPI_LDS = false;
  OccMap occ;
  __host__ __device__ __forceinline__ bool k_list() const { return occ.map != nullptr; }
  // K runs over the destinations, M over the sources
  __device__ __forceinline__ bool k_active(const GemmCtx &x, int m0, int bm, int k0, int bk) const {
    return occ.any(x.z, k0, min(k0 + bk, x.K), m0, min(m0 + bm, x.M));
  }
  RegionView<T> v;
  const T *A;  // [B*R][Dr][lda]
  int lda;
  const T *Os;  // [B][os_rows][C], rows [0, D) already divided by Z
  int os_rows;
  T *Y;
  float *part;
  __device__ __forceinline__ float *split_buffer() const { return part; }
  __device__ __forceinline__ void finish(const GemmCtx &x, int m, int n, f32x4 acc) const {
    store4<T>(Y + ((size_t)x.b * v.N + v.token(x.rho, m)) * v.C + n, acc);
  }
  __device__ __forceinline__ GemmCtx setup(int bz) const {
    return GemmCtx{v.Nr, v.C, v.Dr, bz / v.R, bz % v.R, bz};
  }
  __device__ __forceinline__ bool a_linear(int) const { return true; }
  __device__ __forceinline__ bool b_linear(int) const { return true; }
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &x, int m, int k) const {
    return A + ((size_t)x.z * x.K + k) * lda + m;
  }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &x, int n, int k) const {
    return Os + ((size_t)x.b * os_rows + x.rho * v.Dr + k) * v.C + n;
  }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane, void *wave_lds) const {
    T *out = Y + (size_t)x.b * v.N * v.C;
    const RegionView<T> vv = v;
    const int rr = x.rho;
    store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N,
                  [=](int m) { return out + (size_t)vv.token(rr, m) * vv.C; }, [](int n) { return n; },
                  [](int) { return 1.0f; });
  }
};

// Os[b][j][:] = O[b][j][:] / max(Z[b][j], 1e-20) for the D merged rows of each sample.
template <typename T>
__global__ void k_scale_rows(const T *__restrict__ O, const float *__restrict__ Z, T *__restrict__ Os, int D,
                             int o_rows, int C, size_t total) {
  size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  int cc = (int)(e % C);
  size_t row = e / C;
  int j = (int)(row % D), b = (int)(row / D);
  float rz = 1.0f / fmaxf(Z[(size_t)b * D + j], 1e-20f);
  Os[e] = from_f32<T>(to_f32(O[((size_t)b * o_rows + j) * C + cc]) * rz);
}

// Occupancy map of A (see toma_internal.h).  One workgroup per (WIDE packets of a row, destination
// block, region): the rows of the block stream through 256 / WIDE at a time, every thread ORs the
// raw bits of the packets of its column (eight loads in flight), and the columns of one source
// block are combined through LDS.  (-0 counts as occupied: harmless.)  Narrow pieces of the rows
// and many workgroups suit this read best: 512 bytes per row and workgroup here.
template <int ES, int WIDE>  // WIDE: packets of a row per workgroup
__global__ __launch_bounds__(256) void k_occupancy(const char *__restrict__ A, uint8_t *__restrict__ occ, int Dr,
                                                  int Nr, int occ_db, int occ_sb) {
  constexpr int RG = 256 / WIDE;          // row groups: rows of the block in flight side by side
  constexpr int PPB = kOccSrc * ES / 16;  // packets per source block
  constexpr int NB = WIDE / PPB;          // source blocks per workgroup
  __shared__ uint32_t any[NB];
  const int tid = threadIdx.x, col = tid % WIDE, r2 = tid / WIDE;
  const int z = blockIdx.z, dblk = blockIdx.y;
  const size_t row_bytes = (size_t)Nr * ES;
  const int pkt = blockIdx.x * WIDE + col;  // packet index inside a row
  if (tid < NB) any[tid] = 0;
  __syncthreads();
  uint32_t acc = 0;
  if ((size_t)pkt * 16 < row_bytes) {
    const int j0 = dblk * kOccDest, j1 = min(j0 + kOccDest, Dr);
    const char *base = A + ((size_t)z * Dr) * row_bytes + (size_t)pkt * 16;
    for (int j = j0 + r2; j < j1; j += 8 * RG) {
      u32x4 q[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int jj = min(j + RG * u, j1 - 1);  // (a repeated last row changes nothing)
        q[u] = *reinterpret_cast<const u32x4 *>(base + (size_t)jj * row_bytes);
      }
#pragma unroll
      for (int u = 0; u < 8; u++) acc |= q[u][0] | q[u][1] | q[u][2] | q[u][3];
    }
  }
  if (acc) atomicOr(&any[col / PPB], 1u);
  __syncthreads();
  const int sblk = blockIdx.x * NB + tid;
  if (tid < NB && sblk < occ_sb) occ[((size_t)z * occ_db + dblk) * occ_sb + sblk] = any[tid] ? 1 : 0;
}

int launch_occupancy(const Shape &s, const void *A, uint8_t *occ, const Workspace &w, hipStream_t st) {
  if (w.occ_sb == 0) return TOMA_OK;
  const int es = s.dtype == TOMA_BF16 ? 2 : 4;
  const int row_packets = s.Nr * es / 16;
  constexpr int wide = 32;  // packets of a row per workgroup (128, 64 and 16 measured slower)
  const dim3 grid((row_packets + wide - 1) / wide, w.occ_db, s.B * s.R);
  KernelTimer kt(K_OCC, st);
  const char *Ab = static_cast<const char *>(A);
  if (es == 2)
    hipLaunchKernelGGL((k_occupancy<2, wide>), grid, dim3(256), 0, st, Ab, occ, s.Dr, s.Nr, w.occ_db, w.occ_sb);
  else
    hipLaunchKernelGGL((k_occupancy<4, wide>), grid, dim3(256), 0, st, Ab, occ, s.Dr, s.Nr, w.occ_db, w.occ_sb);
  return launch_status();
}

// Pass 1 of the weights: per source row and slice of destinations (max logit, sum of exponentials),
// then lse[source] = log sum over all destinations.  k_lse also zeroes `zero_words` words at `zero`.
template <typename T>
static GemmShape stats_pass(const Shape &s, const void *X, const int32_t *idx, float2 *stats, int stat_parts, float *lse,
                            float2 *lse2, uint32_t *zero, size_t zero_words, hipStream_t st) {
  WeightsPol<T, false> p1{};
  p1.v = make_view<T>(s, X);
  p1.idx = idx; p1.scale = s.scale;
  p1.stats = stats; p1.parts = stat_parts;
  const int batch = s.B * s.R;
  const GemmShape gs = launch_gemm<T>(K_WSTATS, p1, s.Nr, s.Dr, s.C, batch, st);
  const int rows = batch * s.Nr;
  KernelTimer kt(K_LSE, st);
  hipLaunchKernelGGL(k_lse, dim3((rows + 15) / 16), dim3(256), 0, st, stats, lse, lse2, rows, stat_parts, gs.wgn * gs.tiles_n,
                     zero, zero_words);
  return gs;
}

int launch_weight_stats(const Shape &s, const void *X, const int32_t *idx, float2 *stats, int stat_parts, float *lse,
                        float2 *lse2, int *slice, hipStream_t st) {
  const GemmShape gs = s.dtype == TOMA_BF16 ? stats_pass<bf16_t>(s, X, idx, stats, stat_parts, lse, lse2, nullptr, 0, st)
                                            : stats_pass<float>(s, X, idx, stats, stat_parts, lse, lse2, nullptr, 0, st);
  *slice = gs.bn / gs.wgn;
  if (*slice != weight_stats_slice(s.Nr, s.Dr, s.C, s.B * s.R, s.dtype == TOMA_BF16 ? 2 : 4)) return TOMA_ERR_LAUNCH;
  return launch_status();
}

template <typename T>
static int weights_typed(const Shape &s, const void *X, const int32_t *idx, void *A, float *Z, uint8_t *occ_out,
                         char *ws, const Workspace &w, hipStream_t st) {
  int batch = s.B * s.R;
  const int zr = s.B * s.D;
  // partial row sums of the stored weights, for k_zsum: not needed where the merge product makes Z
  float *zpart = w.z_in_merge ? nullptr : reinterpret_cast<float *>(ws + w.zpart);
  if (weights_single_pass(s.Nr, s.Dr, s.C, batch, (int)sizeof(T))) {
    const RegionView<T> v = make_view<T>(s, X);
    const int tiles = s.Nr / 32;
    const dim3 grid(tiles * batch);
    // the kernel fills the occupancy map itself when a wave's slice of destinations is whole blocks
    const bool own_map = w.occ_sb != 0 && (s.Dr / 8) % kOccDest == 0;
    uint8_t *occ = own_map ? occ_out : nullptr;
    {
      KernelTimer kt(K_WWRITE, st);
      switch (s.Dr / 128) {
#define TOMA_WF_CASE(NJ)                                                                                         \
  case NJ:                                                                                                       \
    hipLaunchKernelGGL((k_weights_fused<T, NJ>), grid, dim3(512), 0, st, v, idx, s.scale, static_cast<T *>(A),   \
                       s.Nr, zpart, w.z_parts, occ, w.occ_db, w.occ_sb, tiles);                                  \
    break;
        TOMA_WF_CASE(1)
        TOMA_WF_CASE(2)
        TOMA_WF_CASE(4)
        TOMA_WF_CASE(8)
        TOMA_WF_CASE(16)
#undef TOMA_WF_CASE
        default: return TOMA_ERR_UNSUPPORTED;
      }
    }
    if (!w.z_in_merge) {  // (else the merge product that follows makes Z from its own A fragments)
      KernelTimer kt(K_ZSUM, st);
      hipLaunchKernelGGL(k_zsum, dim3((zr + 15) / 16), dim3(256), 0, st, zpart, Z, zr, w.z_parts, s.Nr / 32);
    }
    if (launch_status() != TOMA_OK) return TOMA_ERR_LAUNCH;
    return own_map ? TOMA_OK : launch_occupancy(s, A, occ_out, w, st);
  }
  float2 *stats = reinterpret_cast<float2 *>(ws + w.stats);
  float *lse = reinterpret_cast<float *>(ws + w.lse);
  // the write pass fills the occupancy map too (every wave tile lies inside one block of
  // destinations: the wave slices of the planner's tiles divide kOccDest); k_lse zeroes it first
  const bool own_map = w.occ_sb != 0;
  uint8_t *occ = own_map ? occ_out : nullptr;
  const size_t occ_words = own_map ? ((size_t)batch * w.occ_db * w.occ_sb + 3) / 4 : 0;
  const GemmShape gs = stats_pass<T>(s, X, idx, stats, w.stat_parts, lse, nullptr, reinterpret_cast<uint32_t *>(occ), occ_words, st);
  WeightsPol<T, true> p2{};
  p2.v = make_view<T>(s, X); p2.idx = idx; p2.scale = s.scale; p2.lse = lse;
  p2.A = static_cast<T *>(A); p2.lda = s.Nr;
  p2.zpart = zpart; p2.zparts = w.z_parts;
  p2.occ = occ; p2.occ_db = w.occ_db; p2.occ_sb = w.occ_sb;
  // (pass 1 wrote one statistic per wave slice of its tiles: slices of bn / wgn destinations)
  p2.seen = stats; p2.seen_parts = w.stat_parts; p2.slice = gs.bn / gs.wgn;
  const GemmShape gw = launch_gemm<T>(K_WWRITE, p2, s.Nr, s.Dr, s.C, batch, st);
  if (!w.z_in_merge) {
    KernelTimer kt(K_ZSUM, st);
    hipLaunchKernelGGL(k_zsum, dim3((zr + 15) / 16), dim3(256), 0, st, p2.zpart, Z, zr, w.z_parts, gw.wgm * gw.tiles_m);
  }
  return launch_status();
}

int launch_weights(const Shape &s, const void *X, const int32_t *idx, void *A, float *Z, uint8_t *occ, char *ws,
                   const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? weights_typed<bf16_t>(s, X, idx, A, Z, occ, ws, w, st)
                              : weights_typed<float>(s, X, idx, A, Z, occ, ws, w, st);
}

template <typename T>
static int merge_typed(const Shape &s, const void *X, const void *A, float *Z, bool make_z, const uint8_t *occ, void *Xm,
                       char *ws, const Workspace &w, hipStream_t st) {
  MergePol<T> p{};
  p.v = make_view<T>(s, X);
  p.A = static_cast<const T *>(A); p.lda = s.Nr; p.Z = Z; p.Xm = static_cast<T *>(Xm);
  p.Zout = make_z && w.z_in_merge ? Z : nullptr;
  p.occ = OccMap{w.occ_sb ? occ : nullptr, w.occ_db, w.occ_sb};
  p.part = reinterpret_cast<float *>(ws + w.split);
  launch_gemm<T>(K_MERGE, p, s.Dr, s.C, s.Nr, s.B * s.R, st);
  return launch_status();
}

int launch_merge(const Shape &s, const void *X, const void *A, float *Z, bool make_z, const uint8_t *occ, void *Xm,
                 char *ws, const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? merge_typed<bf16_t>(s, X, A, Z, make_z, occ, Xm, ws, w, st)
                              : merge_typed<float>(s, X, A, Z, make_z, occ, Xm, ws, w, st);
}

int launch_scale_rows(const Shape &s, const void *O, const float *Z, int o_rows, void *Os, hipStream_t st) {
  const size_t total = (size_t)s.B * s.D * s.C;
  KernelTimer kt(K_SCALE, st);
  const dim3 grid((unsigned)((total + 255) / 256));
  if (s.dtype == TOMA_BF16)
    hipLaunchKernelGGL(k_scale_rows<bf16_t>, grid, dim3(256), 0, st, static_cast<const bf16_t *>(O), Z,
                       static_cast<bf16_t *>(Os), s.D, o_rows, s.C, total);
  else
    hipLaunchKernelGGL(k_scale_rows<float>, grid, dim3(256), 0, st, static_cast<const float *>(O), Z,
                       static_cast<float *>(Os), s.D, o_rows, s.C, total);
  return launch_status();
}

template <typename T>
static int unmerge_typed(const Shape &s, const void *A, const float *Z, const uint8_t *occ, const void *O, int o_rows,
                         bool prescaled, void *Y, char *ws, const Workspace &w, hipStream_t st) {
  UnmergePol<T> p{};
  if (prescaled) {
    p.Os = static_cast<const T *>(O); p.os_rows = o_rows;
  } else {
    T *Os = reinterpret_cast<T *>(ws + w.os);
    size_t total = (size_t)s.B * s.D * s.C;
    KernelTimer kt(K_SCALE, st);
    hipLaunchKernelGGL(k_scale_rows<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       static_cast<const T *>(O), Z, Os, s.D, o_rows, s.C, total);
    p.Os = Os; p.os_rows = s.D;
  }
  p.v = make_view<T>(s, nullptr);
  p.A = static_cast<const T *>(A); p.lda = s.Nr; p.Y = static_cast<T *>(Y);
  p.occ = OccMap{w.occ_sb ? occ : nullptr, w.occ_db, w.occ_sb};
  p.part = reinterpret_cast<float *>(ws + w.split);
  launch_gemm<T>(K_UNMERGE, p, s.Nr, s.C, s.Dr, s.B * s.R, st);
  return launch_status();
}

int launch_unmerge(const Shape &s, const void *A, const float *Z, const uint8_t *occ, const void *O, int o_rows,
                   bool prescaled, void *Y, char *ws, const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? unmerge_typed<bf16_t>(s, A, Z, occ, O, o_rows, prescaled, Y, ws, w, st)
                              : unmerge_typed<float>(s, A, Z, occ, O, o_rows, prescaled, Y, ws, w, st);
}

}  // namespace toma
