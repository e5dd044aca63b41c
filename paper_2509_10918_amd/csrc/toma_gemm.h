// Block GEMM on the matrix cores with LDS-staged tiles, shared by the merge-weight, merge, QKV /
// output projection and unmerge stages.
//
// Two kernels compute a BM x BN output tile per workgroup from 16 x 16 MFMA tiles, K advancing
// 128 bytes per step (64 bf16 / 32 fp32):
//   k_gemm_async  the main one: 8 waves (4 x 2), tiles from 256 x 256 down to 64 x 64, operand tiles
//                 copied global -> LDS by the load-to-LDS path through a ring of 2-4 stages, one
//                 barrier per step, optional K split between workgroups (see the kernel);
//   k_gemm        the fallback for shapes the ring cannot take (K not a multiple of the step): 4
//                 waves (2 x 2), 128 x 128 / 128 x 64 / 64 x 64, operands staged through registers
//                 into two LDS stages.
// Workgroup ids are remapped so that the tiles an XCD works on are neighbours (they share operand
// rows through that XCD's L2).
//
// An operand is either k-contiguous in memory (a row of the matrix is a run of k: tokens, rows of
// A) or k-major (consecutive k are separate rows and the other index is contiguous: X as the right
// operand of the merge, W[k][n], A as the left operand of the unmerge).  k-contiguous tiles are
// read back as 16-byte fragments; k-major tiles keep their memory order in LDS and are read with
// the LDS transpose read (bf16), so that no operand is ever transposed by a copy.
//
// A policy type describes one product:
//   static constexpr bool A_KS, B_KS      operand is k-major
//   GemmCtx setup(int z) const            decode the batch index into extents M, N, K
//   const T* a_ptr(ctx, int m, int k)     address of element (m, k); the 16-byte packet starting
//   const T* b_ptr(ctx, int n, int k)     there runs along k (k-contiguous) or along m / n (k-major)
//   bool a_linear(int step), b_linear(int step)   address is affine in k over multiples of `step`
//   static constexpr bool ACC_T           accumulator orientation: false = lane holds column
//                                         n_w + 16 j + lane % 16 and rows m_w + 16 i + 4 (lane / 16) + r;
//                                         true = the transposed product (operands swapped in the MFMA):
//                                         lane holds row m_w + 16 i + lane % 16 and the four CONSECUTIVE
//                                         columns n_w + 16 j + 4 (lane / 16) + r, which a row-major
//                                         output stores as one 8- or 16-byte packet
//   void epilogue<TM, TN>(ctx, acc, m_w, n_w, lane, wave_lds)  consume the wave's accumulators
//   static constexpr int EPI              weight of the epilogue in the tile planner's cost model
//   static constexpr bool EPI_LDS         the epilogue wants wave_lds: TM x TN x 256 elements of LDS
//                                         scratch per wave (else it is passed a null pointer)
//   static constexpr bool SPLIT_K         K may be split between workgroups; then also
//   float* split_buffer()                 fp32 partial tiles [split][batch][M][N], and
//   void finish(ctx, m, n, f32x4 v)       output step for four consecutive columns of a summed row
// and optionally (detected by the traits below)
//   static constexpr bool SPARSE_K        with k_list() / k_active(ctx, m0, bm, k0, bk): only the K
//                                         steps the policy calls active are run
//   static constexpr bool EMPTY_TILES     with tile_is_empty() / write_empty_tile(): output tiles the
//                                         policy can prove empty are written without their product
//   static constexpr bool B_STEP_OFFSET   with b_step_uniform() / b_step_offset(ctx, k): a B operand
//                                         that is not affine in k but moves as a whole per K step
// The policy itself is never written to, so it stays in the kernel-argument segment.
// Extents along a packet's direction must be multiples of the packet length (8 bf16 / 4 fp32).
#pragma once
#include <type_traits>

#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

struct GemmCtx { int M, N, K, b, rho, z, split; };

// A policy may declare SPARSE_K = true and supply k_list() / k_active(): the kernel then runs only
// the K steps the policy calls active (see k_gemm_async).
// A policy may also declare EMPTY_TILES = true and supply tile_is_empty() / write_empty_tile(): a
// workgroup whose whole output tile the policy can prove empty writes it without the product.
template <typename P, typename = void> struct PolEmptyTiles { static constexpr bool value = false; };
template <typename P> struct PolEmptyTiles<P, std::void_t<decltype(P::EMPTY_TILES)>> { static constexpr bool value = P::EMPTY_TILES; };
// B_STEP_OFFSET = true with b_step_uniform() / b_step_offset(): a B operand that is not linear in k
// but moves as a whole from one K step to the next.
template <typename P, typename = void> struct PolStepB { static constexpr bool value = false; };
template <typename P> struct PolStepB<P, std::void_t<decltype(P::B_STEP_OFFSET)>> { static constexpr bool value = P::B_STEP_OFFSET; };
template <typename P, typename = void> struct PolRowSums { static constexpr bool value = false; };
template <typename P> struct PolRowSums<P, std::void_t<decltype(P::ROW_SUMS)>> { static constexpr bool value = P::ROW_SUMS; };
template <typename P, typename = void> struct PolSparseK { static constexpr bool value = false; };
template <typename P> struct PolSparseK<P, std::void_t<decltype(P::SPARSE_K)>> { static constexpr bool value = P::SPARSE_K; };

template <typename T, int BM, int BN> struct GemmTile {
  static constexpr int ES = (int)sizeof(T);
  static constexpr int BK = 128 / ES;               // k per step
  static constexpr int KSUB = BK / 32;              // 32-wide MFMA groups per step
  static constexpr int EPP = 16 / ES;               // elements per 16-byte packet
  static constexpr int LDK = BK + EPP;              // k-contiguous tile [rows][BK], padded row
  static constexpr int PADN = 32 / ES;
  static constexpr int TM = BM / 32, TN = BN / 32;  // 16 x 16 MFMA tiles per wave
  static constexpr int NPA = BM / 32, NPB = BN / 32;  // 16-byte packets per thread per operand tile
  static constexpr int a_elems(bool ks) { return ks ? BK * (BM + PADN) : BM * LDK; }
  static constexpr int b_elems(bool ks) { return ks ? BK * (BN + PADN) : BN * LDK; }
};

// rs: row sums of the A operand (one tile per 16 rows, every column of it the same), kept only by
// policies that ask for them (ROW_SUMS)
template <int TM, int TN> struct WaveAccT { f32x4 t[TM][TN]; f32x4 rs[TM]; };

// K split between workgroups: the raw fp32 accumulators go to part[split][z][M][N].
template <bool ACC_T, int TM, int TN>
__device__ __forceinline__ void store_partial(float *part, const GemmCtx &x, const WaveAccT<TM, TN> &acc, int nbatch,
                                              int m_w, int n_w, int lane) {
  const int g = lane >> 4, c = lane & 15;
  float *base = part + ((size_t)x.split * nbatch + x.z) * x.M * x.N;
  if constexpr (ACC_T) {
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const int m = m_w + 16 * i + c;
      if (m >= x.M) continue;
#pragma unroll
      for (int j = 0; j < TN; j++) {
        const int n = n_w + 16 * j + 4 * g;
        if (n < x.N) *reinterpret_cast<f32x4 *>(base + (size_t)m * x.N + n) = acc.t[i][j];
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int m = m_w + 16 * i + 4 * g + r;
        if (m >= x.M) continue;
#pragma unroll
        for (int j = 0; j < TN; j++) {
          const int n = n_w + 16 * j + c;
          if (n < x.N) base[(size_t)m * x.N + n] = acc.t[i][j][r];
        }
      }
  }
}

template <typename T, typename Pol, int BM, int BN>
__global__ __launch_bounds__(256) void k_gemm(const Pol pol, int tiles_m, int tiles_n) {
  typedef GemmTile<T, BM, BN> G;
  constexpr int A_ELEMS = G::a_elems(Pol::A_KS), B_ELEMS = G::b_elems(Pol::B_KS);
  constexpr int LDA = Pol::A_KS ? BM + G::PADN : G::LDK;
  constexpr int LDB = Pol::B_KS ? BN + G::PADN : G::LDK;
  __shared__ __align__(16) T As[2][A_ELEMS];
  __shared__ __align__(16) T Bs[2][B_ELEMS];

  int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int per_batch = tiles_m * tiles_n;
  const int z = tile / per_batch;
  tile -= z * per_batch;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const GemmCtx ctx = pol.setup(z);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
  const int g = lane >> 4, c = lane & 15;
  const int K = ctx.K;

  // where this thread's packets sit inside a tile
  int a_lds[G::NPA], a_i[G::NPA], a_k[G::NPA], b_lds[G::NPB], b_i[G::NPB], b_k[G::NPB];
#pragma unroll
  for (int i = 0; i < G::NPA; i++) {
    int q = tid + 256 * i;
    if (Pol::A_KS) {
      constexpr int PPN = BM / G::EPP;
      a_k[i] = q / PPN; a_i[i] = (q % PPN) * G::EPP; a_lds[i] = a_k[i] * LDA + a_i[i];
    } else {
      constexpr int PPR = G::BK / G::EPP;
      a_i[i] = q / PPR; a_k[i] = (q % PPR) * G::EPP; a_lds[i] = a_i[i] * LDA + a_k[i];
    }
  }
#pragma unroll
  for (int i = 0; i < G::NPB; i++) {
    int q = tid + 256 * i;
    if (Pol::B_KS) {
      constexpr int PPN = BN / G::EPP;
      b_k[i] = q / PPN; b_i[i] = (q % PPN) * G::EPP; b_lds[i] = b_k[i] * LDB + b_i[i];
    } else {
      constexpr int PPR = G::BK / G::EPP;
      b_i[i] = q / PPR; b_k[i] = (q % PPR) * G::EPP; b_lds[i] = b_i[i] * LDB + b_k[i];
    }
  }

  WaveAccT<G::TM, G::TN> acc;
#pragma unroll
  for (int i = 0; i < G::TM; i++)
#pragma unroll
    for (int j = 0; j < G::TN; j++) acc.t[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  Pkt ra[G::NPA], rb[G::NPB];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < G::NPA; i++) {
      int m = m0 + a_i[i], ka = k0 + a_k[i];
      ra[i] = (m < ctx.M && ka < K) ? pkt_load(pol.a_ptr(ctx, m, ka)) : pkt_zero();
    }
#pragma unroll
    for (int i = 0; i < G::NPB; i++) {
      int n = n0 + b_i[i], kb = k0 + b_k[i];
      rb[i] = (n < ctx.N && kb < K) ? pkt_load(pol.b_ptr(ctx, n, kb)) : pkt_zero();
    }
  };
  auto stash = [&](int stage) {
#pragma unroll
    for (int i = 0; i < G::NPA; i++) pkt_store(As[stage] + a_lds[i], ra[i]);
#pragma unroll
    for (int i = 0; i < G::NPB; i++) pkt_store(Bs[stage] + b_lds[i], rb[i]);
  };

  fetch(0);
  stash(0);
  __syncthreads();
  int stage = 0;
  for (int k0 = 0; k0 < K; k0 += G::BK) {
    const bool more = k0 + G::BK < K;
    if (more) fetch(k0 + G::BK);
    const T *at = As[stage], *bt = Bs[stage];
#pragma unroll
    for (int kk = 0; kk < G::KSUB; kk++) {
      Frag<T> fa[G::TM], fb[G::TN];
      const int kf = 32 * kk + 8 * g;
#pragma unroll
      for (int i = 0; i < G::TM; i++) {
        const int row = wm * (BM / 2) + 16 * i;
        if (Pol::A_KS) frag_load_ks(fa[i], at, LDA, kf, kf + 4, row, lane);
        else frag_load_kc(fa[i], at + (row + c) * LDA + kf);
      }
#pragma unroll
      for (int j = 0; j < G::TN; j++) {
        const int col = wn * (BN / 2) + 16 * j;
        if (Pol::B_KS) frag_load_ks(fb[j], bt, LDB, kf, kf + 4, col, lane);
        else frag_load_kc(fb[j], bt + (col + c) * LDB + kf);
      }
#pragma unroll
      for (int i = 0; i < G::TM; i++)
#pragma unroll
        for (int j = 0; j < G::TN; j++) {
          if constexpr (Pol::ACC_T) mma16(acc.t[i][j], fb[j], fa[i]);
          else mma16(acc.t[i][j], fa[i], fb[j]);
        }
    }
    if (more) stash(stage ^ 1);
    __syncthreads();
    stage ^= 1;
  }

  pol.template epilogue<G::TM, G::TN>(ctx, acc, m0 + wm * (BM / 2), n0 + wn * (BN / 2), lane, nullptr);
}

// ------------------------------------------------------------------------------------------------
// The same product with the operand tiles copied global -> LDS by the load-to-LDS path
// (global_load_lds, 16 bytes per lane, no register staging) through a ring of STAGES tiles, so that
// several K steps of loads are in flight while the matrix cores work on the oldest one.
// A load-to-LDS instruction writes lane l's 16 bytes at (LDS base + 16 l): LDS tiles are therefore
// dense 1 KiB chunks, and bank conflicts are avoided by permuting WHICH global packet a lane
// fetches (an XOR swizzle of the packet index by the row), undone by the fragment reads.
// Needs K to be a multiple of the K step; rows past the end are clamped (their results are never
// stored).  Other shapes use k_gemm above.
// ------------------------------------------------------------------------------------------------
template <typename T> struct SwzTile {
  static constexpr int ES = (int)sizeof(T);
  static constexpr int EPP = 16 / ES;
  // k-contiguous tile: 128-byte rows of 8 packets; packet kp of row r sits at slot kp ^ (r & 7)
  __device__ static __forceinline__ int kc(int row, int kp) { return row * (128 / ES) + ((kp ^ (row & 7)) * EPP); }
  // k-contiguous tile with rows of PPR >= 8 packets: the same swizzle inside each group of 8
  template <int PPR> __device__ static __forceinline__ int kcw(int row, int kp) {
    return (row * PPR + ((kp & ~7) | ((kp ^ row) & 7))) * EPP;
  }
  // k-major tile: rows of PPR packets; packet pi of row k sits at slot ks_slot(k, pi).  A transpose
  // read touches, per 16 lanes, four consecutive k-rows x 32 bytes: the low bits of k spread them
  // over one 128-byte bank group; bit 3 of k (the second 16 lanes of each half wave sit eight rows
  // further) selects the other 128-byte group when a row is long enough to have one.
  // G4: the second 16 lanes sit FOUR rows further (the attention kernel's key order).  A long row
  // again has its other 128-byte group for them; with 128-byte rows, where odd and even rows already
  // alternate between the two groups, they take the 32-byte pieces that the first 16 lanes leave free.
  template <int PPR, bool G4 = false> __device__ static __forceinline__ int ks_slot(int k, int pi) {
    if constexpr (G4) {
      if (PPR >= 16) return pi ^ ((k & 3) << 1) ^ (((k >> 2) & 1) << 3);
      return pi ^ (((k & 3) ^ ((k >> 2) & 1)) << 1);
    }
    int s = pi ^ ((k & 3) << 1);
    if (PPR >= 16) s ^= ((k >> 3) & 1) << 3;
    return s;
  }
  template <int PPR, bool G4 = false> __device__ static __forceinline__ int ks(int k, int pi) {
    return (k * PPR + ks_slot<PPR, G4>(k, pi)) * EPP;
  }
};

template <int PPR, bool G4 = false>
__device__ __forceinline__ void frag_load_ks_sw(Frag<bf16_t> &f, const bf16_t *tile, int ka, int kb, int nb, int lane) {
  typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const int j = lane & 15, col = nb + 4 * (j & 3);
  const int ra = ka + (j >> 2), rb = kb + (j >> 2);
  const bf16_t *pa = tile + SwzTile<bf16_t>::ks<PPR, G4>(ra, col >> 3) + (col & 7);
  const bf16_t *pb = tile + SwzTile<bf16_t>::ks<PPR, G4>(rb, col >> 3) + (col & 7);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(pa));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(pb));
  s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  f.v = __builtin_bit_cast(bf16x8, both);
}
template <int PPR, bool G4 = false>
__device__ __forceinline__ void frag_load_ks_sw(Frag<float> &f, const float *tile, int ka, int kb, int nb, int lane) {
  const int col = nb + (lane & 15);
#pragma unroll
  for (int i = 0; i < 4; i++) {
    f.v[i] = tile[SwzTile<float>::ks<PPR, G4>(ka + i, col >> 2) + (col & 3)];
    f.v[4 + i] = tile[SwzTile<float>::ks<PPR, G4>(kb + i, col >> 2) + (col & 3)];
  }
}
// eight consecutive k starting at element kf of row `row` of a swizzled k-contiguous tile
__device__ __forceinline__ void frag_load_kc_sw(Frag<bf16_t> &f, const bf16_t *tile, int row, int kf) {
  f.v = *reinterpret_cast<const bf16x8 *>(tile + SwzTile<bf16_t>::kc(row, kf >> 3));
}
__device__ __forceinline__ void frag_load_kc_sw(Frag<float> &f, const float *tile, int row, int kf) {
  f32x4 a = *reinterpret_cast<const f32x4 *>(tile + SwzTile<float>::kc(row, kf >> 2));
  f32x4 b = *reinterpret_cast<const f32x4 *>(tile + SwzTile<float>::kc(row, (kf >> 2) + 1));
#pragma unroll
  for (int i = 0; i < 4; i++) { f.v[i] = a[i]; f.v[4 + i] = b[i]; }
}

// eight consecutive k starting at element kf of a row of PPR packets
template <int PPR> __device__ __forceinline__ void frag_load_kcw_sw(Frag<bf16_t> &f, const bf16_t *tile, int row, int kf) {
  f.v = *reinterpret_cast<const bf16x8 *>(tile + SwzTile<bf16_t>::kcw<PPR>(row, kf >> 3));
}
template <int PPR> __device__ __forceinline__ void frag_load_kcw_sw(Frag<float> &f, const float *tile, int row, int kf) {
  f32x4 a = *reinterpret_cast<const f32x4 *>(tile + SwzTile<float>::kcw<PPR>(row, kf >> 2));
  f32x4 b = *reinterpret_cast<const f32x4 *>(tile + SwzTile<float>::kcw<PPR>(row, (kf >> 2) + 1));
#pragma unroll
  for (int i = 0; i < 4; i++) { f.v[i] = a[i]; f.v[4 + i] = b[i]; }
}

// One load-to-LDS instruction: lane l's 16 bytes at gptr land at lds_chunk + 16 l.  Issued as
// assembly so that the pipeline's own s_waitcnt vmcnt(n) (below) decides when a tile is complete;
// the compiler's model would otherwise drain every outstanding load before each LDS read.
template <typename T>
__device__ __forceinline__ void load_to_lds16(const T *gptr, T *lds_chunk) {
  uint32_t lds_addr = (uint32_t)(size_t)(__attribute__((address_space(3))) void *)lds_chunk;
  lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr)
               : "memory", "m0");
}
// The same with the LDS byte address already in a scalar register (see lds_addr_of): pipelines
// that compute their ring addresses once keep the per-load cost at the M0 write and the load.
__device__ __forceinline__ uint32_t lds_addr_of(const void *lds_ptr) {
  const uint32_t a = (uint32_t)(size_t)(__attribute__((address_space(3))) const void *)lds_ptr;
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)a);
}
template <typename T>
__device__ __forceinline__ void load_to_lds16_at(const T *gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr)
               : "memory", "m0");
}
// The same from a wave-uniform base (scalar registers) plus a per-lane byte offset (32 bits, unsigned):
// a pipeline whose lanes keep fixed offsets inside a tile then spends no vector instruction on addresses.
template <typename T>
__device__ __forceinline__ void load_to_lds16_from(const T *uniform_base, uint32_t lane_bytes, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_bytes), "s"(uniform_base)
               : "memory", "m0");
}
// wait until at most n of this wave's vector-memory loads are outstanding (n < 64)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 0xf) | (((N >> 4) & 3) << 14));
}

// Workgroup: 8 waves as 4 x 2, two waves per SIMD (a single wave cannot keep a matrix core busy:
// operand fetch and execution of successive MFMAs only overlap across waves).  With bf16 a K step
// has two 32-wide sub-steps and the fragment reads run one sub-step ahead of the products, so the
// LDS latency hides behind the matrix cores; the single barrier of a step sits between its two
// halves, after this wave's last read of the current stage and before its first read of the next.
// nsplit > 1 splits K between workgroups; their fp32 partial tiles are combined by k_split_finish.
template <typename T, typename Pol, int BM, int BN, int STAGES, int WAVES = 8>
__global__ __launch_bounds__(64 * WAVES) void k_gemm_async(const Pol pol, int tiles_m, int tiles_n, int nbatch, int nsplit) {
  typedef GemmTile<T, BM, BN> G;
  constexpr int WGM = WAVES == 4 ? 2 : 4, WGN = WAVES / WGM, NWAVES = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;               // wave tile
  constexpr int TM = WTM / 16, TN = WTN / 16;                 // 16 x 16 MFMA tiles per wave
  constexpr int A_ELEMS = BM * G::BK, B_ELEMS = BN * G::BK;   // dense: 128 bytes per row / k-row
  constexpr int NIA = BM / 8 / NWAVES, NIB = BN / 8 / NWAVES; // load instructions per wave per tile
  constexpr int PPR_A = BM / G::EPP, PPR_B = BN / G::EPP;     // packets per k-row of a k-major tile
  __shared__ __align__(1024) T As[STAGES][A_ELEMS];
  __shared__ __align__(1024) T Bs[STAGES][B_ELEMS];

  int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int per_batch = tiles_m * tiles_n;
  const int zs = tile / per_batch;
  tile -= zs * per_batch;
  const int z = zs / nsplit, split = zs - z * nsplit;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  GemmCtx ctx = pol.setup(z);
  ctx.split = split;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w / WGN, wn = w % WGN;
  const int g = lane >> 4, c = lane & 15;
  if constexpr (PolEmptyTiles<Pol>::value) {
    // every thread checks its share of the evidence; all must agree
    if (__syncthreads_and(pol.tile_is_empty(ctx, m0, n0, BM, BN, tid, 64 * WAVES) ? 1 : 0)) {
      pol.write_empty_tile(ctx, m0, n0, BM, BN, BM / WGM, tid, 64 * WAVES);
      return;
    }
  }
  // this workgroup's share of the K steps
  const int nk_all = ctx.K / G::BK;
  const int kt0 = (int)((long long)nk_all * split / nsplit), kt1 = (int)((long long)nk_all * (split + 1) / nsplit);
  int nk = kt1 - kt0;
  const int kbase = kt0 * G::BK;

  // Sparse K: wave 0 asks the policy about every K step of this workgroup's range and compacts the
  // active ones into a list; the pipeline below then walks the list instead of the range.  Each
  // wave keeps the current 64 entries of the list in one register (entry i in lane i % 64).
  constexpr bool kSparse = PolSparseK<Pol>::value;
  constexpr int kMaxList = kSparse ? 1024 : 1;
  __shared__ uint16_t klist[kMaxList];
  __shared__ int klist_n;
  bool listed = false;
  if constexpr (kSparse) {
    if (pol.k_list() && nk <= kMaxList) {
      if (w == 0) {
        int count = 0;
        for (int c0 = 0; c0 < nk; c0 += 64) {
          const int kt = c0 + lane;
          const bool act = kt < nk && pol.k_active(ctx, m0, BM, kbase + kt * G::BK, G::BK);
          const uint64_t mask = __ballot(act);
          if (act) klist[count + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)kt;
          count += __popcll(mask);
        }
        if (lane == 0) klist_n = count;
      }
      __syncthreads();
      nk = klist_n;
      listed = true;
    }
  }
  uint32_t kreg = 0;  // list entries 64 c + lane of the chunk c the issue index is in
  auto list_chunk = [&](int j) {
    if constexpr (kSparse) {
      if (listed) { const int e = (j & ~63) + lane; kreg = e < nk ? klist[e] : 0; }
    }
  };
  // K step that issue index j stands for
  auto step_of = [&](int j) -> int {
    if constexpr (kSparse) {
      if (listed) {
        if ((j & 63) == 0 && j > 0) list_chunk(j);
        return __builtin_amdgcn_readlane((int)kreg, j & 63);
      }
    }
    return j;
  };
  list_chunk(0);

  // what this lane fetches for chunk `ch` (1 KiB = 64 packets) of a tile: tile coordinates
  int a_i[NIA], a_k[NIA], b_i[NIB], b_k[NIB];
#pragma unroll
  for (int t = 0; t < NIA; t++) {
    const int ch = w * NIA + t;
    if (Pol::A_KS) {
      const int k = ch * (64 / PPR_A) + lane / PPR_A, pos = lane % PPR_A;
      a_k[t] = k; a_i[t] = SwzTile<T>::template ks_slot<PPR_A>(k, pos) * G::EPP;
    } else {
      const int row = ch * 8 + (lane >> 3);
      a_i[t] = row; a_k[t] = ((lane & 7) ^ (row & 7)) * G::EPP;
    }
    // rows past the end repeat the last valid row / packet
    const int lim = Pol::A_KS ? ctx.M - G::EPP : ctx.M - 1;
    if (m0 + a_i[t] > lim) a_i[t] = lim - m0;
  }
#pragma unroll
  for (int t = 0; t < NIB; t++) {
    const int ch = w * NIB + t;
    if (Pol::B_KS) {
      const int k = ch * (64 / PPR_B) + lane / PPR_B, pos = lane % PPR_B;
      b_k[t] = k; b_i[t] = SwzTile<T>::template ks_slot<PPR_B>(k, pos) * G::EPP;
    } else {
      const int row = ch * 8 + (lane >> 3);
      b_i[t] = row; b_k[t] = ((lane & 7) ^ (row & 7)) * G::EPP;
    }
    const int lim = Pol::B_KS ? ctx.N - G::EPP : ctx.N - 1;
    if (n0 + b_i[t] > lim) b_i[t] = lim - n0;
  }

  // Operand addresses advance by a fixed amount per K step when the operand is linear in k (all
  // operands except a k-major walk over a region whose width does not divide the step): keep the
  // first step's address and the per-step delta instead of recomputing maps and gathers every step.
  const bool lin_a = pol.a_linear(G::BK), lin_b = pol.b_linear(G::BK);
  const T *pa[NIA], *pb[NIB];
#pragma unroll
  for (int t = 0; t < NIA; t++) pa[t] = pol.a_ptr(ctx, m0 + a_i[t], kbase + a_k[t]);
#pragma unroll
  for (int t = 0; t < NIB; t++) pb[t] = pol.b_ptr(ctx, n0 + b_i[t], kbase + b_k[t]);
  // the per-step delta of a linear operand is the same for every packet: keep it in a scalar register
  const int da = lin_a ? __builtin_amdgcn_readfirstlane((int)(pol.a_ptr(ctx, m0 + a_i[0], kbase + a_k[0] + G::BK) - pa[0])) : 0;
  const int db = lin_b ? __builtin_amdgcn_readfirstlane((int)(pol.b_ptr(ctx, n0 + b_i[0], kbase + b_k[0] + G::BK) - pb[0])) : 0;
  // (a B operand that moves as a whole per step: one wave-uniform offset per step instead of an
  // address computation per packet)
  bool step_b = false;
  ptrdiff_t step_b0 = 0;
  if constexpr (PolStepB<Pol>::value) {
    step_b = !lin_b && pol.b_step_uniform(G::BK);
    if (step_b) step_b0 = pol.b_step_offset(ctx, kbase);
  }
  const bool b_fast = lin_b || step_b;
  // Ring positions are passed down as plain integers.  For all but the largest tile the K loop
  // below is unrolled by the number of stages, which makes them constants after inlining: the LDS
  // addresses of the loads are then scalar constants off one base, and the fragment reads use
  // fixed offsets off a few per-lane bases instead of being recomputed every step.  (The
  // 256 x 256 tile has no registers to spare for per-stage bases and keeps a rolled loop.)
  constexpr bool kUnroll = BM * BN <= 256 * 128;
  // Reading the fragments one sub-step ahead needs a second set of fragment registers.  The largest
  // tile cannot afford them when exactly one operand is k-major (measured: the spills cost more than
  // the exposed LDS latency, which the SIMD's other wave covers).
  constexpr bool kPipelineFrags = kUnroll || Pol::A_KS == Pol::B_KS;
  const uint32_t w_s = (uint32_t)__builtin_amdgcn_readfirstlane(w);
  const uint32_t a_lds = lds_addr_of(&As[0][0]) + w_s * (NIA * 1024);
  const uint32_t b_lds = lds_addr_of(&Bs[0][0]) + w_s * (NIB * 1024);
  auto issue = [&](int st, int j) {
    const int kt = step_of(j);
    const int k0 = kbase + kt * G::BK;
    const uint32_t a_st = a_lds + (uint32_t)st * (A_ELEMS * G::ES), b_st = b_lds + (uint32_t)st * (B_ELEMS * G::ES);
#pragma unroll
    for (int t = 0; t < NIA; t++) {
      const T *src = lin_a ? pa[t] + (ptrdiff_t)kt * da : pol.a_ptr(ctx, m0 + a_i[t], k0 + a_k[t]);
      load_to_lds16_at(src, a_st + (uint32_t)(t * 1024));
    }
    // one wave-uniform offset per step covers the linear and the step-uniform case alike
    ptrdiff_t b_off = (ptrdiff_t)kt * db;
    if constexpr (PolStepB<Pol>::value) {
      if (step_b) b_off = pol.b_step_offset(ctx, k0) - step_b0;
    }
#pragma unroll
    for (int t = 0; t < NIB; t++) {
      const T *src = b_fast ? pb[t] + b_off : pol.b_ptr(ctx, n0 + b_i[t], k0 + b_k[t]);
      load_to_lds16_at(src, b_st + (uint32_t)(t * 1024));
    }
  };
  // this wave's loads of step kt are the oldest outstanding ones: wait until at most the younger
  // steps' loads remain
  auto wait_stage = [&](int kt) {
    const int younger = min(nk - 1 - kt, STAGES - 2);
    if (STAGES >= 4 && younger >= 2) wait_vmcnt<2 * (NIA + NIB)>();
    else if (STAGES >= 3 && younger >= 1) wait_vmcnt<NIA + NIB>();
    else wait_vmcnt<0>();
  };
  // workgroup barrier that the compiler may not move memory accesses across
  auto meet = [&]() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  auto frags = [&](Frag<T> (&fa)[TM], Frag<T> (&fb)[TN], int st, int kk) {
    const T *at = As[st], *bt = Bs[st];
    const int kf = 32 * kk + 8 * g;
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const int row = wm * WTM + 16 * i;
      if (Pol::A_KS) frag_load_ks_sw<PPR_A>(fa[i], at, kf, kf + 4, row, lane);
      else frag_load_kc_sw(fa[i], at, row + c, kf);
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int col = wn * WTN + 16 * j;
      if (Pol::B_KS) frag_load_ks_sw<PPR_B>(fb[j], bt, kf, kf + 4, col, lane);
      else frag_load_kc_sw(fb[j], bt, col + c, kf);
    }
  };

  WaveAccT<TM, TN> acc;
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) acc.t[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  // Row sums of A on the side (a policy's choice per launch): one more product per A fragment, against a
  // fragment of ones - in the transposed orientation every lane then holds the sum of the row it stores.
  bool row_sums = false;
  Frag<T> ones;
  if constexpr (PolRowSums<Pol>::value) {
    static_assert(Pol::ACC_T && !Pol::A_KS, "row sums are kept in the transposed orientation of a k-contiguous A");
    row_sums = pol.row_sums();
#pragma unroll
    for (int e = 0; e < 8; e++) ones.v[e] = from_f32<T>(1.0f);
#pragma unroll
    for (int i = 0; i < TM; i++) acc.rs[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }
  auto products = [&](const Frag<T> (&fa)[TM], const Frag<T> (&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        if constexpr (Pol::ACC_T) mma16(acc.t[i][j], fb[j], fa[i]);
        else mma16(acc.t[i][j], fa[i], fb[j]);
      }
    if constexpr (PolRowSums<Pol>::value) {
      if (row_sums) {
#pragma unroll
        for (int i = 0; i < TM; i++) mma16(acc.rs[i], ones, fa[i]);
      }
    }
  };
  auto next_stage = [](int st) { return st + 1 == STAGES ? 0 : st + 1; };
  auto prev_stage = [](int st) { return st == 0 ? STAGES - 1 : st - 1; };
  // runs step(st, kt) for kt = 0 .. nk - 1 with st = kt % STAGES
  auto k_loop = [&](auto &&step) {
    if constexpr (kUnroll) {
      for (int kt = 0; kt < nk; kt += STAGES) {
        step(0, kt);
        if constexpr (STAGES >= 2) { if (kt + 1 < nk) step(1, kt + 1); }
        if constexpr (STAGES >= 3) { if (kt + 2 < nk) step(2, kt + 2); }
        if constexpr (STAGES >= 4) { if (kt + 3 < nk) step(3, kt + 3); }
      }
    } else {
      for (int kt = 0, st = 0; kt < nk; kt++, st = next_stage(st)) step(st, kt);
    }
  };

  // prologue: the loads of the first STAGES - 1 steps
#pragma unroll
  for (int s = 0; s < STAGES - 1; s++)
    if (s < nk) issue(s, s);

  if constexpr (G::KSUB == 2 && kPipelineFrags) {
    Frag<T> fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    wait_stage(0);
    meet();
    frags(fa0, fb0, 0, 0);
    k_loop([&](int st, int kt) {
      // every wave is past the barrier of step kt - 1: the stage of step kt - 1 is free
      if (kt + STAGES - 1 < nk) issue(prev_stage(st), kt + STAGES - 1);
      frags(fa1, fb1, st, 1);
      products(fa0, fb0);
      if (kt + 1 < nk) wait_stage(kt + 1);
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's reads of stage kt have returned
      meet();
      if (kt + 1 < nk) frags(fa0, fb0, next_stage(st), 0);
      products(fa1, fb1);
    });
  } else {
    k_loop([&](int st, int kt) {
      wait_stage(kt);
      // every wave's part of tile kt has landed, and every wave is done reading tile kt - 1
      meet();
      if (kt + STAGES - 1 < nk) issue(prev_stage(st), kt + STAGES - 1);
#pragma unroll
      for (int kk = 0; kk < G::KSUB; kk++) {
        Frag<T> fa[TM], fb[TN];
        frags(fa, fb, st, kk);
        products(fa, fb);
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);
    });
  }

  if constexpr (Pol::SPLIT_K) {
    if (nsplit > 1) {
      store_partial<Pol::ACC_T, TM, TN>(pol.split_buffer(), ctx, acc, nbatch, m0 + wm * WTM, n0 + wn * WTN, lane);
      return;
    }
  }
  // an epilogue that asked for it gets a share of the (now idle) operand tiles as scratch, one
  // element per accumulator value of the wave: all waves inside the A tiles when those are large
  // enough, else half of the waves in the A tiles and half in the B tiles
  void *wave_lds = nullptr;
  if constexpr (Pol::EPI_LDS) {
    constexpr int kWave = WTM * WTN;
    if constexpr (STAGES * A_ELEMS >= NWAVES * kWave) {
      meet();  // every wave is done reading the tiles
      wave_lds = &As[0][0] + w * kWave;
    } else if constexpr (STAGES * A_ELEMS >= NWAVES / 2 * kWave && STAGES * B_ELEMS >= NWAVES / 2 * kWave) {
      meet();
      wave_lds = w < NWAVES / 2 ? &As[0][0] + w * kWave : &Bs[0][0] + (w - NWAVES / 2) * kWave;
    }
  }
  pol.template epilogue<TM, TN>(ctx, acc, m0 + wm * WTM, n0 + wn * WTN, lane, wave_lds);
}

// four consecutive output elements as one store
template <typename T> __device__ __forceinline__ void store4(T *dst, f32x4 v) {
  alignas(16) T o[4];
#pragma unroll
  for (int i = 0; i < 4; i++) o[i] = from_f32<T>(v[i]);
  if (sizeof(T) == 2) *reinterpret_cast<u32x2 *>(dst) = *reinterpret_cast<u32x2 *>(o);
  else *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<u32x4 *>(o);
}

// Row-major store of a wave's TRANSPOSED accumulators (ACC_T): the four consecutive columns a lane
// holds of row m go to row(m) + col(n) as one packet, scaled per row.  col(n) .. col(n) + 3 must be
// contiguous for n a multiple of 4, and N a multiple of 4.
struct ElemIdentity { __device__ __forceinline__ f32x4 operator()(f32x4 v) const { return v; } };
template <typename T, int TM, int TN, typename RowFn, typename ColFn, typename RowScaleFn, typename ElemFn = ElemIdentity>
__device__ __forceinline__ void store_rows(const WaveAccT<TM, TN> &acc, int m_w, int n_w, int lane, int M, int N,
                                           RowFn row, ColFn col, RowScaleFn row_scale, ElemFn elem = ElemFn()) {
  const int g = lane >> 4, c = lane & 15;
  // the column parts once, outside the rows' conditional code (left inside, each row's copy of a
  // column offset that needs a division is computed again)
  decltype(col(0)) coff[TN];
#pragma unroll
  for (int j = 0; j < TN; j++) coff[j] = col(n_w + 16 * j + 4 * g);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int m = m_w + 16 * i + c;
    if (m >= M) continue;
    T *base = row(m);
    const float sc = row_scale(m);
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n_w + 16 * j + 4 * g;
      if (n < N) store4<T>(base + coff[j], elem(acc.t[i][j] * sc));
    }
  }
}

// Sum of the K-split partial tiles in a fixed order, then the policy's own output step.  One thread
// per four consecutive columns.
template <typename T, typename Pol>
__global__ __launch_bounds__(256) void k_split_finish(const Pol pol, int nbatch, int nsplit) {
  const int z = blockIdx.y;
  GemmCtx ctx = pol.setup(z);
  ctx.split = 0;
  const int n4 = ctx.N >> 2;
  const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= (size_t)ctx.M * n4) return;
  const int m = (int)(q / n4), n = (int)(q % n4) * 4;
  const float *part = pol.split_buffer();
  f32x4 v = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < nsplit; s++)
    v += *reinterpret_cast<const f32x4 *>(part + (((size_t)s * nbatch + z) * ctx.M + m) * ctx.N + n);
  pol.finish(ctx, m, n, v);
}

struct GemmShape { int bm, bn, wgm, wgn, tiles_m, tiles_n, nsplit; };

inline GemmShape make_gemm_shape(int M, int N, int bm, int bn, int wgm, int wgn) {
  return GemmShape{bm, bn, wgm, wgn, (M + bm - 1) / bm, (N + bn - 1) / bn, 1};
}

// Tile shape for the register-staged kernel: the largest that still gives about two workgroups per CU.
inline GemmShape choose_gemm_shape(int M, int N, int batch) {
  auto blocks = [&](const GemmShape &g) { return (long long)g.tiles_m * g.tiles_n * batch; };
  GemmShape g = make_gemm_shape(M, N, 128, 128, 2, 2);
  if (blocks(g) >= 512) return g;
  g = make_gemm_shape(M, N, 128, 64, 2, 2);
  if (blocks(g) >= 512) return g;
  return make_gemm_shape(M, N, 64, 64, 2, 2);
}

// Width (in columns) of one wave's slice of the block tile that launch_gemm picks for a product that
// may not split K: the granularity of per-slice results such as the weights' statistics.
inline int weight_stats_slice(int M, int N, int K, int batch, int elem_size) {
  if (gemm_async_fits(M, N, K, elem_size)) return plan_gemm_async(M, N, K, batch, elem_size, false, false, false, 3).bn / 2;
  return choose_gemm_shape(M, N, batch).bn / 2;
}

template <typename T, typename Pol>
inline GemmShape launch_gemm(int kernel_id, const Pol &pol, int M, int N, int K, int batch, hipStream_t st) {
  if (gemm_async_fits(M, N, K, (int)sizeof(T))) {
    // load-to-LDS pipeline
    GemmPlan pl;
    if constexpr (PolSparseK<Pol>::value) {
      static_assert(Pol::SPLIT_K && Pol::EPI == 1, "map products are planned by plan_map_product");
      pl = plan_map_product(M, N, K, batch, (int)sizeof(T), Pol::A_KS, Pol::B_KS, pol.k_list());
    } else {
      pl = plan_gemm_async(M, N, K, batch, (int)sizeof(T), Pol::SPLIT_K, Pol::A_KS, Pol::B_KS, Pol::EPI);
    }
    const GemmShape g{pl.bm, pl.bn, 4, 2, (M + pl.bm - 1) / pl.bm, (N + pl.bn - 1) / pl.bn, pl.nsplit};
    const dim3 grid(g.tiles_m * g.tiles_n * batch * g.nsplit);
    {
      KernelTimer kt(kernel_id, st);
      if (g.bm == 256 && g.bn == 256)
        hipLaunchKernelGGL((k_gemm_async<T, Pol, 256, 256, 2>), grid, dim3(512), 0, st, pol, g.tiles_m, g.tiles_n, batch, g.nsplit);
      else if (g.bm == 256)
        hipLaunchKernelGGL((k_gemm_async<T, Pol, 256, 128, 3>), grid, dim3(512), 0, st, pol, g.tiles_m, g.tiles_n, batch, g.nsplit);
      else if (g.bm == 128 && g.bn == 128)
        hipLaunchKernelGGL((k_gemm_async<T, Pol, 128, 128, 4>), grid, dim3(512), 0, st, pol, g.tiles_m, g.tiles_n, batch, g.nsplit);
      else if (g.bm == 128)
        hipLaunchKernelGGL((k_gemm_async<T, Pol, 128, 64, 4>), grid, dim3(512), 0, st, pol, g.tiles_m, g.tiles_n, batch, g.nsplit);
      else
        hipLaunchKernelGGL((k_gemm_async<T, Pol, 64, 64, 4>), grid, dim3(512), 0, st, pol, g.tiles_m, g.tiles_n, batch, g.nsplit);
    }
    if constexpr (Pol::SPLIT_K) if (g.nsplit > 1) {
      KernelTimer kt(K_SPLIT, st);
      const size_t quads = (size_t)M * (N / 4);
      hipLaunchKernelGGL((k_split_finish<T, Pol>), dim3((unsigned)((quads + 255) / 256), batch), dim3(256), 0, st, pol,
                         batch, g.nsplit);
    }
    return g;
  }
  const GemmShape g = choose_gemm_shape(M, N, batch);
  const dim3 grid(g.tiles_m * g.tiles_n * batch);
  KernelTimer kt(kernel_id, st);
  if (g.bm == 128 && g.bn == 128)
    hipLaunchKernelGGL((k_gemm<T, Pol, 128, 128>), grid, dim3(256), 0, st, pol, g.tiles_m, g.tiles_n);
  else if (g.bm == 128)
    hipLaunchKernelGGL((k_gemm<T, Pol, 128, 64>), grid, dim3(256), 0, st, pol, g.tiles_m, g.tiles_n);
  else
    hipLaunchKernelGGL((k_gemm<T, Pol, 64, 64>), grid, dim3(256), 0, st, pol, g.tiles_m, g.tiles_n);
  return g;
}

}  // namespace toma
