// Block GEMM on the matrix cores with LDS-staged tiles, shared by the merge-weight, merge, QKV /
// output projection and unmerge stages.  One workgroup (4 waves, 2 x 2) computes a 128 x 128
// output tile; each wave owns 64 x 64 as 4 x 4 MFMA tiles; K advances 32 per step with the next
// step's global loads issued before the current step's products.
//
// An operand is either k-contiguous in memory (a row of the matrix is a run of k: tokens, weight
// rows of A) or k-major (consecutive k are separate rows and the other index is contiguous: X as
// the right operand of the merge, W[k][n], A as the left operand of the unmerge).  k-contiguous
// tiles are read back as 16-byte fragments; k-major tiles keep their memory order in LDS and are
// read with the LDS transpose read (bf16) so that no operand is ever transposed by a copy.
//
// A policy type describes one product:
//   static constexpr bool A_KS, B_KS      operand is k-major
//   GemmCtx setup(int z) const            decode the batch index blockIdx.z into extents M, N, K
//   const T* a_ptr(ctx, int m, int k)     address of element (m, k); the 16-byte packet starting
//   const T* b_ptr(ctx, int n, int k)     there runs along k (k-contiguous) or along m / n (k-major)
//   void epilogue(ctx, acc, m_w, n_w, lane)  consume the wave's 64 x 64 accumulators
// The policy itself is never written to, so it stays in the kernel-argument segment.
// Extents along a packet's direction must be multiples of the packet length (8 bf16 / 4 fp32).
#pragma once
#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

template <typename T> struct GemmTile {
  static constexpr int BM = 128, BN = 128, BK = 32;
  static constexpr int EPP = 16 / (int)sizeof(T);  // elements per 16-byte packet
  static constexpr int LDK = BK + EPP;             // row stride of a k-contiguous tile [128][BK]
  static constexpr int LDN = 128 + EPP;            // row stride of a k-major tile [BK][128]
  static constexpr int KC_ELEMS = 128 * LDK;
  static constexpr int KS_ELEMS = BK * LDN;
  static constexpr int NP = 128 * BK / EPP / 256;  // packets per thread per operand tile
};

typedef f32x4 WaveAcc[4][4];

struct GemmCtx { int M, N, K, b, rho, z; };

template <typename T, typename Pol>
__global__ __launch_bounds__(256) void k_gemm(const Pol pol) {
  typedef GemmTile<T> G;
  constexpr int A_ELEMS = Pol::A_KS ? G::KS_ELEMS : G::KC_ELEMS;
  constexpr int B_ELEMS = Pol::B_KS ? G::KS_ELEMS : G::KC_ELEMS;
  __shared__ __align__(16) T As[A_ELEMS];
  __shared__ __align__(16) T Bs[B_ELEMS];

  const GemmCtx ctx = pol.setup(blockIdx.z);
  const int m0 = blockIdx.y * G::BM, n0 = blockIdx.x * G::BN;
  if (m0 >= ctx.M || n0 >= ctx.N) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
  const int g = lane >> 4, c = lane & 15;
  const int K = ctx.K;

  // where this thread's packets sit inside a tile
  int a_lds[G::NP], a_i[G::NP], a_k[G::NP], b_lds[G::NP], b_i[G::NP], b_k[G::NP];
#pragma unroll
  for (int i = 0; i < G::NP; i++) {
    int q = tid + 256 * i;
    if (Pol::A_KS) {
      constexpr int PPN = 128 / G::EPP;
      a_k[i] = q / PPN; a_i[i] = (q % PPN) * G::EPP; a_lds[i] = a_k[i] * G::LDN + a_i[i];
    } else {
      constexpr int PPR = G::BK / G::EPP;
      a_i[i] = q / PPR; a_k[i] = (q % PPR) * G::EPP; a_lds[i] = a_i[i] * G::LDK + a_k[i];
    }
    if (Pol::B_KS) {
      constexpr int PPN = 128 / G::EPP;
      b_k[i] = q / PPN; b_i[i] = (q % PPN) * G::EPP; b_lds[i] = b_k[i] * G::LDN + b_i[i];
    } else {
      constexpr int PPR = G::BK / G::EPP;
      b_i[i] = q / PPR; b_k[i] = (q % PPR) * G::EPP; b_lds[i] = b_i[i] * G::LDK + b_k[i];
    }
  }

  WaveAcc acc;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  Pkt ra[G::NP], rb[G::NP];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < G::NP; i++) {
      int m = m0 + a_i[i], ka = k0 + a_k[i];
      ra[i] = (m < ctx.M && ka < K) ? pkt_load(pol.a_ptr(ctx, m, ka)) : pkt_zero();
      int n = n0 + b_i[i], kb = k0 + b_k[i];
      rb[i] = (n < ctx.N && kb < K) ? pkt_load(pol.b_ptr(ctx, n, kb)) : pkt_zero();
    }
  };

  fetch(0);
  for (int k0 = 0; k0 < K; k0 += G::BK) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < G::NP; i++) {
      pkt_store(As + a_lds[i], ra[i]);
      pkt_store(Bs + b_lds[i], rb[i]);
    }
    __syncthreads();
    if (k0 + G::BK < K) fetch(k0 + G::BK);

    Frag<T> fa[4], fb[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if (Pol::A_KS) frag_load_ks(fa[i], As, G::LDN, 8 * g, 8 * g + 4, wm * 64 + 16 * i, lane);
      else frag_load_kc(fa[i], As + (wm * 64 + 16 * i + c) * G::LDK + 8 * g);
      if (Pol::B_KS) frag_load_ks(fb[i], Bs, G::LDN, 8 * g, 8 * g + 4, wn * 64 + 16 * i, lane);
      else frag_load_kc(fb[i], Bs + (wn * 64 + 16 * i + c) * G::LDK + 8 * g);
    }
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) mma16(acc[i][j], fa[i], fb[j]);
  }

  pol.epilogue(ctx, acc, m0 + wm * 64, n0 + wn * 64, lane);
}

// Row-major store of a wave's accumulators: element (m, n) goes to ptr(m, n), scaled per row.
// ptr must be contiguous in n inside an aligned run of 16 columns.
template <typename T, typename PtrFn, typename RowScaleFn>
__device__ __forceinline__ void store_rows(const WaveAcc &acc, int m_w, int n_w, int lane, int M, int N,
                                           PtrFn ptr, RowScaleFn row_scale) {
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      int m = m_w + 16 * i + 4 * g + r;
      if (m >= M) continue;
      float sc = row_scale(m);
#pragma unroll
      for (int j = 0; j < 4; j++) {
        int n = n_w + 16 * j + c;
        if (n < N) *ptr(m, n) = from_f32<T>(acc[i][j][r] * sc);
      }
    }
}

template <typename T, typename Pol>
inline void launch_gemm(int kernel_id, const Pol &pol, int M, int N, int batch, hipStream_t st) {
  dim3 grid((N + 127) / 128, (M + 127) / 128, batch);
  KernelTimer kt(kernel_id, st);
  hipLaunchKernelGGL((k_gemm<T, Pol>), grid, dim3(256), 0, st, pol);
}

}  // namespace toma
