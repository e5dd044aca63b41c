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
#include "toma_gemm.h"
#include "toma_internal.h"

namespace toma {

template <typename T> struct RegionView {
  const T *X;
  RegionMap map;
  int N, C, D, R, Nr, Dr;
  __device__ __forceinline__ int token(int rho, int s) const { return R == 1 ? s : map.token(rho, s); }
  // token(rho, s + step) - token(rho, s) does not depend on s
  __device__ __forceinline__ bool token_linear(int step) const { return R == 1 || step % map.tile_w == 0; }
};

// ---- pass 1 and pass 2 of the weights ----------------------------------------------------------
template <typename T, bool WRITE> struct WeightsPol {
  static constexpr bool A_KS = false, B_KS = false, SPLIT_K = false, ACC_T = false;
  static constexpr int EPI = 3;
  RegionView<T> v;
  const int32_t *idx;
  float scale;
  float2 *stats;   // pass 1 out: [B*R][Nr][parts]
  int parts;
  const float *lse;  // pass 2 in: [B*R][Nr]
  T *A;              // pass 2 out: [B*R][Dr][lda], lda >= Nr
  int lda;
  float *zpart;      // pass 2 out: [B*R][Dr][zparts]
  int zparts;
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
                                           int lane) const {
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
            colsum[j] += to_f32(o[r]);
          }
          T *dst = A + ((size_t)z * N + n) * lda + mb;
          if (sizeof(T) == 2) {
            *reinterpret_cast<u32x2 *>(dst) = *reinterpret_cast<u32x2 *>(o);
          } else {
            *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<u32x4 *>(o);
          }
        }
      }
      const int part = m_w / (16 * TM);
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
};

// lse[row] = M + log(sum_i s_i exp(m_i - M)) over the row's partial (max, sum) pairs.  One 16-lane
// group per row, partials strided over its lanes; the combination order is fixed.
__global__ __launch_bounds__(256) void k_lse(const float2 *__restrict__ stats, float *__restrict__ lse, int rows,
                                            int stride, int parts) {
  int row = (blockIdx.x * 256 + threadIdx.x) >> 4, c = threadIdx.x & 15;
  if (row >= rows) return;
  const float2 *s = stats + (size_t)row * stride;
  float mx = -__builtin_inff();
  for (int i = c; i < parts; i += 16) mx = fmaxf(mx, s[i].x);
  mx = row16_max_f32(mx);
  float sum = 0.f;
  for (int i = c; i < parts; i += 16) sum += s[i].y * __expf(s[i].x - mx);
  sum = row16_sum_f32(sum);
  if (c == 0) lse[row] = mx + __logf(sum);
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

// ---- merge -------------------------------------------------------------------------------------
template <typename T> struct MergePol {
  static constexpr bool A_KS = false, B_KS = true, SPLIT_K = true, ACC_T = true;
  static constexpr int EPI = 1;
  RegionView<T> v;
  const T *A;  // [B*R][Dr][lda]
  int lda;
  const float *Z;
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
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &x, int m, int k) const {
    return A + ((size_t)x.z * x.M + m) * lda + k;
  }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &x, int n, int k) const {
    return v.X + ((size_t)x.b * v.N + v.token(x.rho, k)) * v.C + n;
  }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane) const {
    const float *Zr = Z + (size_t)x.b * v.D + x.rho * v.Dr;
    T *out = Xm + ((size_t)x.b * v.D + x.rho * v.Dr) * v.C;
    const int Cc = v.C;
    store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N,
                  [=](int m) { return out + (size_t)m * Cc; }, [](int n) { return n; },
                  [=](int m) { return 1.0f / fmaxf(Zr[m], 1e-20f); });
  }
};

// ---- unmerge -----------------------------------------------------------------------------------
template <typename T> struct UnmergePol {
  static constexpr bool A_KS = true, B_KS = true, SPLIT_K = true, ACC_T = true;
  static constexpr int EPI = 1;
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
                                           int lane) const {
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

template <typename T>
__global__ void k_copy_extra(const T *__restrict__ O, T *__restrict__ Ye, int D, int T_extra, int C, size_t total) {
  size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  size_t per = (size_t)T_extra * C;
  size_t b = e / per, r = e % per;
  Ye[e] = O[(b * (size_t)(D + T_extra) + D) * C + r];
}

template <typename T> static RegionView<T> make_view(const Shape &s, const void *X) {
  RegionView<T> v;
  v.X = static_cast<const T *>(X);
  v.map = RegionMap{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  v.N = s.N; v.C = s.C; v.D = s.D; v.R = s.R; v.Nr = s.Nr; v.Dr = s.Dr;
  return v;
}

template <typename T>
static int weights_typed(const Shape &s, const void *X, const int32_t *idx, void *A, float *Z, char *ws,
                         const Workspace &w, hipStream_t st) {
  int batch = s.B * s.R;
  WeightsPol<T, false> p1{};
  p1.v = make_view<T>(s, X);
  p1.idx = idx; p1.scale = s.scale;
  p1.stats = reinterpret_cast<float2 *>(ws + w.stats); p1.parts = w.stat_parts;
  const GemmShape gs = launch_gemm<T>(K_WSTATS, p1, s.Nr, s.Dr, s.C, batch, st);
  float *lse = reinterpret_cast<float *>(ws + w.lse);
  int rows = batch * s.Nr;
  { KernelTimer kt(K_LSE, st);
    hipLaunchKernelGGL(k_lse, dim3((rows + 15) / 16), dim3(256), 0, st, p1.stats, lse, rows, w.stat_parts, gs.wgn * gs.tiles_n); }
  WeightsPol<T, true> p2{};
  p2.v = p1.v; p2.idx = idx; p2.scale = s.scale; p2.lse = lse;
  p2.A = static_cast<T *>(A); p2.lda = s.Nr;
  p2.zpart = reinterpret_cast<float *>(ws + w.zpart); p2.zparts = w.z_parts;
  const GemmShape gw = launch_gemm<T>(K_WWRITE, p2, s.Nr, s.Dr, s.C, batch, st);
  int zr = s.B * s.D;
  { KernelTimer kt(K_ZSUM, st);
    hipLaunchKernelGGL(k_zsum, dim3((zr + 15) / 16), dim3(256), 0, st, p2.zpart, Z, zr, w.z_parts, gw.wgm * gw.tiles_m); }
  return launch_status();
}

int launch_weights(const Shape &s, const void *X, const int32_t *idx, void *A, float *Z, char *ws,
                   const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? weights_typed<bf16_t>(s, X, idx, A, Z, ws, w, st)
                              : weights_typed<float>(s, X, idx, A, Z, ws, w, st);
}

template <typename T>
static int merge_typed(const Shape &s, const void *X, const void *A, const float *Z, void *Xm, char *ws,
                       const Workspace &w, hipStream_t st) {
  MergePol<T> p{};
  p.v = make_view<T>(s, X);
  p.A = static_cast<const T *>(A); p.lda = s.Nr; p.Z = Z; p.Xm = static_cast<T *>(Xm);
  p.part = reinterpret_cast<float *>(ws + w.split);
  launch_gemm<T>(K_MERGE, p, s.Dr, s.C, s.Nr, s.B * s.R, st);
  return launch_status();
}

int launch_merge(const Shape &s, const void *X, const void *A, const float *Z, void *Xm, char *ws,
                 const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? merge_typed<bf16_t>(s, X, A, Z, Xm, ws, w, st)
                              : merge_typed<float>(s, X, A, Z, Xm, ws, w, st);
}

template <typename T>
static int unmerge_typed(const Shape &s, const void *A, const float *Z, const void *O, int o_rows, bool prescaled,
                         void *Y, char *ws, const Workspace &w, hipStream_t st) {
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
  p.part = reinterpret_cast<float *>(ws + w.split);
  launch_gemm<T>(K_UNMERGE, p, s.Nr, s.C, s.Dr, s.B * s.R, st);
  return launch_status();
}

int launch_unmerge(const Shape &s, const void *A, const float *Z, const void *O, int o_rows, bool prescaled,
                   void *Y, char *ws, const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? unmerge_typed<bf16_t>(s, A, Z, O, o_rows, prescaled, Y, ws, w, st)
                              : unmerge_typed<float>(s, A, Z, O, o_rows, prescaled, Y, ws, w, st);
}

int launch_copy_extra(const Shape &s, const void *O, void *Y_extra, hipStream_t st) {
  size_t total = (size_t)s.B * s.T * s.C;
  if (total == 0) return TOMA_OK;
  dim3 grid((unsigned)((total + 255) / 256));
  KernelTimer kt(K_COPY, st);
  if (s.dtype == TOMA_BF16)
    hipLaunchKernelGGL(k_copy_extra<bf16_t>, grid, dim3(256), 0, st, static_cast<const bf16_t *>(O),
                       static_cast<bf16_t *>(Y_extra), s.D, s.T, s.C, total);
  else
    hipLaunchKernelGGL(k_copy_extra<float>, grid, dim3(256), 0, st, static_cast<const float *>(O),
                       static_cast<float *>(Y_extra), s.D, s.T, s.C, total);
  return launch_status();
}

}  // namespace toma
