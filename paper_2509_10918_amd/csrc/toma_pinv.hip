// Moore-Penrose unmerge (paper Sec. 4.2.2, first display): Y = A~^+ X' with A~ = A / Z the
// row-normalised merge matrix of a merge region (Dr destinations x Nr sources, Dr <= 128) and A~^+ its
// pseudo-inverse with singular values <= rcond * largest treated as zero.  The paper measures this
// against the transpose unmerge and rejects it for its cost; it is here so that the comparison can be
// made on this hardware too.
//
//   A~^+ = A~^T (A~ A~^T)^+ :  G = A~ A~^T is Dr x Dr, symmetric, positive semi-definite.
//   k_pinv_eig    one workgroup per (sample, merge region): G in double precision in LDS, its
//                 eigen-decomposition G = V diag(lambda) V^T by cyclic Jacobi rotations (every
//                 sweep rotates all pairs, 64 disjoint pairs at a time in round-robin order), then
//                 G^+ = sum over lambda_k > rcond^2 lambda_max of v_k v_k^T / lambda_k  (lambda =
//                 sigma^2, so this is the singular-value rule).  Rank deficiency of any kind - rows of
//                 A~ that are zero because nobody chose a destination, duplicated or nearly dependent
//                 rows - ends up as eigenvalues below the cut.
//   k_pinv_apply  one workgroup per (region, 32 channels): w = G^+ X' (double), then
//                 Y[token(s)] = sum_j A_js w_j / Z_j, written at the tokens' grid positions.
// Everything between the stored operands and the rounding of Y is double precision: the merge
// matrices of a small temperature have a few singular values of 1e-4 ... 1e-12 next to a bulk in
// [0.2, 1], and the cut has to tell them apart.
#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

constexpr int kPinvMax = 128;            // destinations per merge region this path takes
constexpr int kPinvThreads = 1024;
constexpr int kPinvChunk = 16;           // sources per staging step of G = A A^T

template <typename T> struct PinvView {
  const T *A;          // [B*R][Dr][Nr]
  const float *Z;      // [B][D]
  RegionMap map;
  int N, C, D, R, Nr, Dr, n_loc;
  // grid index of source s of merge region rho (sources region by region, local order inside)
  __device__ __forceinline__ int token(int rho, int s) const {
    return R != 1 ? map.token(rho, s) : map.token(s / n_loc, s % n_loc);
  }
};

__device__ __forceinline__ double block_sum(double v, double *red, int tid, int nthreads) {
  v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64);
  v += __shfl_xor(v, 8, 64); v += __shfl_xor(v, 16, 64); v += __shfl_xor(v, 32, 64);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  double s = 0.0;
  for (int i = 0; i < nthreads / 64; i++) s += red[i];  // fixed order
  return s;
}

template <typename T>
__global__ __launch_bounds__(kPinvThreads) void k_pinv_eig(const PinvView<T> v, double rcond, double *__restrict__ Vt_all,
                                                          double *__restrict__ Ginv_all) {
  // G with a padded row stride (column walks of the rotations would otherwise hit one bank)
  extern __shared__ __align__(16) double lds[];
  const int n = v.Dr, LD = n + 1;
  double *G = lds;                               // [n][LD]
  double *stage = G + (size_t)n * LD;            // [n][kPinvChunk] weights of the current sources, as doubles
  double *rot = stage + (size_t)n * kPinvChunk;  // [n / 2 + 1][4]: p, q, c, s of the round's rotations
  double *red = rot + 4 * (n / 2 + 1);           // [kPinvThreads / 64]
  const int tid = threadIdx.x, z = blockIdx.x, b = z / v.R, rho = z % v.R;
  const T *A = v.A + (size_t)z * n * v.Nr;
  const float *Zr = v.Z + (size_t)b * v.D + (size_t)rho * n;
  double *Vt = Vt_all + (size_t)z * n * n, *Ginv = Ginv_all + (size_t)z * n * n;

  // ---- G = diag(1/Z) A A^T diag(1/Z) ----
  for (int e = tid; e < n * n; e += kPinvThreads) G[(e / n) * LD + e % n] = 0.0;
  for (int s0 = 0; s0 < v.Nr; s0 += kPinvChunk) {
    __syncthreads();
    for (int e = tid; e < n * kPinvChunk; e += kPinvThreads) {
      const int j = e / kPinvChunk, s = s0 + e % kPinvChunk;
      stage[e] = s < v.Nr ? (double)to_f32(A[(size_t)j * v.Nr + s]) : 0.0;
    }
    __syncthreads();
    for (int e = tid; e < n * n; e += kPinvThreads) {
      const int i = e / n, j = e % n;
      if (j < i) continue;  // upper triangle; mirrored below
      double acc = 0.0;
#pragma unroll
      for (int s = 0; s < kPinvChunk; s++) acc += stage[i * kPinvChunk + s] * stage[j * kPinvChunk + s];
      G[i * LD + j] += acc;
    }
  }
  __syncthreads();
  for (int e = tid; e < n * n; e += kPinvThreads) {
    const int i = e / n, j = e % n;
    if (j < i) continue;
    const double g = G[i * LD + j] / ((double)fmaxf(Zr[i], 1e-20f) * (double)fmaxf(Zr[j], 1e-20f));
    G[i * LD + j] = g;
    G[j * LD + i] = g;
  }
  for (int e = tid; e < n * n; e += kPinvThreads) Vt[e] = (e / n == e % n) ? 1.0 : 0.0;
  __syncthreads();

  // ---- cyclic Jacobi: G <- J^T G J, V <- V J for every pair (p, q), until the off-diagonal part is gone ----
  const int np = n + (n & 1), m = np - 1, half = np / 2;  // an odd n plays against a dummy that never rotates
  for (int sweep = 0; sweep < 40; sweep++) {
    double off = 0.0, dia = 0.0;
    for (int e = tid; e < n * n; e += kPinvThreads) {
      const int i = e / n, j = e % n;
      const double g = G[i * LD + j];
      if (i == j) dia += g * g; else off += g * g;
    }
    off = block_sum(off, red, tid, kPinvThreads);
    dia = block_sum(dia, red, tid, kPinvThreads);
    if (off <= 1e-26 * dia || dia == 0.0) break;  // uniform: every thread holds the same sums
    for (int r = 0; r < m; r++) {
      if (tid < half) {
        int p = tid == 0 ? m : (r + tid) % m, q = (r - tid + m) % m;
        double c = 1.0, s = 0.0;
        if (p < n && q < n) {
          const double apq = G[p * LD + q], app = G[p * LD + p], aqq = G[q * LD + q];
          if (fabs(apq) > 1e-300 && fabs(apq) > 1e-20 * sqrt(fabs(app * aqq))) {
            const double th = (aqq - app) / (2.0 * apq);
            const double t = (th >= 0.0 ? 1.0 : -1.0) / (fabs(th) + sqrt(th * th + 1.0));
            c = 1.0 / sqrt(t * t + 1.0);
            s = t * c;
          }
        } else {
          p = q = 0;
        }
        rot[4 * tid + 0] = (double)p; rot[4 * tid + 1] = (double)q; rot[4 * tid + 2] = c; rot[4 * tid + 3] = s;
      }
      __syncthreads();
      // rows p and q of every pair: G <- J^T G
      for (int e = tid; e < half * n; e += kPinvThreads) {
        const int k = e / n, j = e % n;
        const double s = rot[4 * k + 3];
        if (s == 0.0) continue;
        const int p = (int)rot[4 * k], q = (int)rot[4 * k + 1];
        const double c = rot[4 * k + 2], gp = G[p * LD + j], gq = G[q * LD + j];
        G[p * LD + j] = c * gp - s * gq;
        G[q * LD + j] = s * gp + c * gq;
      }
      __syncthreads();
      // columns p and q: G <- G J; the same rotation on the eigenvector rows of V^T
      for (int e = tid; e < half * n; e += kPinvThreads) {
        const int k = e / n, i = e % n;
        const double s = rot[4 * k + 3];
        if (s == 0.0) continue;
        const int p = (int)rot[4 * k], q = (int)rot[4 * k + 1];
        const double c = rot[4 * k + 2], gp = G[i * LD + p], gq = G[i * LD + q];
        G[i * LD + p] = c * gp - s * gq;
        G[i * LD + q] = s * gp + c * gq;
        const double vp = Vt[p * n + i], vq = Vt[q * n + i];
        Vt[p * n + i] = c * vp - s * vq;
        Vt[q * n + i] = s * vp + c * vq;
      }
      __syncthreads();
    }
  }

  // ---- G^+ = sum over the eigenvalues above the cut of v_k v_k^T / lambda_k ----
  double lmax = 0.0;
  for (int k = 0; k < n; k++) lmax = fmax(lmax, G[k * LD + k]);
  const double cut = rcond * rcond * lmax;
  __syncthreads();  // (the rotations' last global writes of V^T are visible to the whole workgroup)
  for (int k = tid; k < n; k += kPinvThreads) {
    const double l = G[k * LD + k];
    stage[k] = (l > cut && l > 0.0) ? 1.0 / l : 0.0;
  }
  __threadfence_block();
  __syncthreads();
  for (int e = tid; e < n * n; e += kPinvThreads) {
    const int i = e / n, j = e % n;
    double acc = 0.0;
    for (int k = 0; k < n; k++) acc += Vt[k * n + i] * Vt[k * n + j] * stage[k];
    Ginv[e] = acc;
  }
}

constexpr int kPinvCols = 32;  // channels per workgroup of the apply kernel

template <typename T>
__global__ __launch_bounds__(256) void k_pinv_apply(const PinvView<T> v, const double *__restrict__ Ginv_all,
                                                   const T *__restrict__ O, int o_rows, T *__restrict__ Y) {
  __shared__ double xs[kPinvMax][kPinvCols + 1];  // X' chunk, then w = G^+ X' / Z in its place
  const int n = v.Dr, tid = threadIdx.x;
  const int z = blockIdx.y, b = z / v.R, rho = z % v.R, c0 = blockIdx.x * kPinvCols;
  const double *Ginv = Ginv_all + (size_t)z * n * n;
  const float *Zr = v.Z + (size_t)b * v.D + (size_t)rho * n;
  for (int e = tid; e < n * kPinvCols; e += 256) {
    const int j = e / kPinvCols, c = e % kPinvCols;
    xs[j][c] = c0 + c < v.C ? (double)to_f32(O[((size_t)b * o_rows + (size_t)rho * n + j) * v.C + c0 + c]) : 0.0;
  }
  __syncthreads();
  constexpr int kPer = kPinvMax * kPinvCols / 256;  // entries of w per thread
  double wv[kPer];
#pragma unroll
  for (int u = 0; u < kPer; u++) {
    const int e = tid + 256 * u, i = e / kPinvCols, c = e % kPinvCols;
    double acc = 0.0;
    if (i < n)
      for (int j = 0; j < n; j++) acc += Ginv[(size_t)i * n + j] * xs[j][c];
    wv[u] = i < n ? acc / (double)fmaxf(Zr[i], 1e-20f) : 0.0;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kPer; u++) {
    const int e = tid + 256 * u, i = e / kPinvCols, c = e % kPinvCols;
    if (i < n) xs[i][c] = wv[u];
  }
  __syncthreads();
  const T *A = v.A + (size_t)z * n * v.Nr;
  // a thread takes a source and eight channels: consecutive threads read consecutive weights of a row of A
  for (int e = tid; e < v.Nr * (kPinvCols / 8); e += 256) {
    const int s = e % v.Nr, cg = (e / v.Nr) * 8;
    double acc[8];
#pragma unroll
    for (int u = 0; u < 8; u++) acc[u] = 0.0;
    for (int j = 0; j < n; j++) {
      const double a = (double)to_f32(A[(size_t)j * v.Nr + s]);
      if (a == 0.0) continue;
#pragma unroll
      for (int u = 0; u < 8; u++) acc[u] += a * xs[j][cg + u];
    }
    T *dst = Y + ((size_t)b * v.N + v.token(rho, s)) * v.C + c0 + cg;
#pragma unroll
    for (int u = 0; u < 8; u++)
      if (c0 + cg + u < v.C) dst[u] = from_f32<T>((float)acc[u]);
  }
}

size_t pinv_workspace_bytes(const Shape &s) {
  if (s.Dr > kPinvMax) return 0;
  return (size_t)2 * s.B * s.R * s.Dr * s.Dr * sizeof(double);
}

template <typename T>
static int pinv_typed(const Shape &s, const void *A, const float *Z, const void *O, int o_rows, float rcond, void *Y,
                      char *ws, const Workspace &w, hipStream_t st) {
  PinvView<T> v;
  v.A = static_cast<const T *>(A); v.Z = Z;
  v.map = RegionMap{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  v.N = s.N; v.C = s.C; v.D = s.D; v.R = s.R; v.Nr = s.Nr; v.Dr = s.Dr; v.n_loc = s.n_loc;
  double *Vt = reinterpret_cast<double *>(ws + w.pinv);
  double *Ginv = Vt + (size_t)s.B * s.R * s.Dr * s.Dr;
  const int n = s.Dr;
  const size_t lds = sizeof(double) * ((size_t)n * (n + 1) + (size_t)n * kPinvChunk + 4 * (n / 2 + 1) + kPinvThreads / 64);
  auto *kern = k_pinv_eig<T>;
  // (more than 64 KiB of dynamic LDS has to be granted per kernel)
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
      hipSuccess)
    return TOMA_ERR_LAUNCH;
  {
    KernelTimer kt(K_PINV_EIG, st);
    hipLaunchKernelGGL(kern, dim3(s.B * s.R), dim3(kPinvThreads), lds, st, v, (double)rcond, Vt, Ginv);
  }
  {
    KernelTimer kt(K_PINV_APPLY, st);
    hipLaunchKernelGGL((k_pinv_apply<T>), dim3((s.C + kPinvCols - 1) / kPinvCols, s.B * s.R), dim3(256), 0, st, v, Ginv,
                       static_cast<const T *>(O), o_rows, static_cast<T *>(Y));
  }
  return launch_status();
}

int launch_unmerge_pinv(const Shape &s, const void *A, const float *Z, const void *O, int o_rows, float rcond, void *Y,
                        char *ws, const Workspace &w, hipStream_t st) {
  if (s.Dr > kPinvMax) return TOMA_ERR_UNSUPPORTED;
  return s.dtype == TOMA_BF16 ? pinv_typed<bf16_t>(s, A, Z, O, o_rows, rcond, Y, ws, w, st)
                              : pinv_typed<float>(s, A, Z, O, o_rows, rcond, Y, ws, w, st);
}

}  // namespace toma
