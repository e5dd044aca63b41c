// The core module on the merged tokens: multi-head scaled dot-product attention (paper Eq. 1 with
// tau = 1; Alg. 3 "computational layer"), on U = [X_merged ; X_extra].
//
//   k_gemm<QkvPol>   Q, K, V = U W  (one launch, blockIdx.z picks the weight), written head-major
//                    [B][heads][L][head_dim] so that every head is a dense matrix.
//   k_attn_async     flash-style attention: 16 queries per wave, four to twelve waves per workgroup
//                    (chosen per launch), 64 keys per step through a ring of K / V tiles in LDS,
//                    online softmax, nothing of size L x L ever stored.  (k_attn: the same with
//                    register-staged tiles, for head widths whose ring does not fit.)
//                    The score tile is computed TRANSPOSED (keys x queries): its accumulator
//                    layout (lane = query, registers = 4 consecutive keys) is then already the
//                    B-operand layout of the second product O^T += V^T P^T, so probabilities go
//                    from accumulators straight back into the matrix cores without touching LDS.
//                    V^T fragments come from the row-major V tile through the LDS transpose read.
//   k_gemm<ProjPol>  optional output projection.
#include <type_traits>

#include "toma_gemm.h"
#include "toma_internal.h"

namespace toma {

template <typename T> struct QkvPol {
  static constexpr bool A_KS = false, B_KS = true, SPLIT_K = false, ACC_T = true;
  static constexpr int EPI = 1;
  static constexpr bool EPI_LDS = false;
  const T *Xm, *Xe;
  const T *W[3];
  T *out[3];
  int B, D, Tx, L, C, H, dh, dh_sh;  // dh_sh = log2(dh), or -1 if dh is not a power of two
  int Kin;                           // width of the input rows (C for self-attention; the context's for cross-attention keys / values)
  __device__ __forceinline__ GemmCtx setup(int bz) const { return GemmCtx{B * L, C, Kin, 0, 0, bz}; }
  __device__ __forceinline__ bool a_linear(int) const { return true; }
  __device__ __forceinline__ bool b_linear(int) const { return true; }
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &, int m, int k) const {
    int b = m / L, l = m % L;
    return l < D ? Xm + ((size_t)b * D + l) * Kin + k : Xe + ((size_t)b * Tx + (l - D)) * Kin + k;
  }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &x, int n, int k) const {
    return W[x.z] + (size_t)k * C + n;
  }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane, void *wave_lds) const {
    // head-major output [B][H][L][dh]: a row's part and a column's part of the offset add up
    // (divisions are dear here: the head width is a power of two, and the sample of a row follows
    // from the sample of the wave tile's first row, which is the same for all lanes)
    T *o = out[x.z];
    const int L_ = L, H_ = H, dh_ = dh, sh = dh_sh;
    const int b0 = m_w / L_, l0 = m_w - b0 * L_;
    store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N,
                  [=](int m) {
                    int b = b0, l = l0 + (m - m_w);
                    if (L_ >= 16 * TM) { if (l >= L_) { l -= L_; b++; } }  // a tile of 16 TM rows crosses one boundary at most
                    else { b = m / L_; l = m - b * L_; }
                    return o + ((size_t)b * H_ * L_ + l) * dh_;
                  },
                  [=](int n) { const int h = sh >= 0 ? n >> sh : n / dh_; return (size_t)h * L_ * dh_ + (n - h * dh_); },
                  [](int) { return 1.0f; });
  }
};

template <typename T> struct ProjPol {
  static constexpr bool A_KS = false, B_KS = true, SPLIT_K = false, ACC_T = true;
  static constexpr int EPI = 1;
  static constexpr bool EPI_LDS = false;
  const T *In, *Wt;
  T *Out;
  const float *Zs;  // when set: rows l < D of every sample are divided by max(Z, 1e-20)
  T *Oe;            // when set: rows l >= D (the extra tokens) go to Oe[b][l - D] instead of Out[b][l]
  int rows, C, L, D;
  __device__ __forceinline__ GemmCtx setup(int) const { return GemmCtx{rows, C, C, 0, 0, 0}; }
  __device__ __forceinline__ bool a_linear(int) const { return true; }
  __device__ __forceinline__ bool b_linear(int) const { return true; }
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &, int m, int k) const { return In + (size_t)m * C + k; }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &, int n, int k) const { return Wt + (size_t)k * C + n; }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane, void *wave_lds) const {
    T *o = Out, *oe = Oe;
    const int C_ = C, L_ = L, D_ = D;
    const float *zs = Zs;
    store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N,
                          [=](int m) {
                            const int b = m / L_, l = m - b * L_;
                            return (oe && l >= D_) ? oe + ((size_t)b * (L_ - D_) + (l - D_)) * C_ : o + (size_t)m * C_;
                          },
                          [](int n) { return n; },
                          [=](int m) {
                            int b = m / L_, l = m % L_;
                            return (zs && l < D_) ? 1.0f / fmaxf(zs[(size_t)b * D_ + l], 1e-20f) : 1.0f;
                          });
  }
};

// Out = act(In W) for a dense [rows, K] x [K, N] product (the feed-forward core module).
struct ElemGelu {  // gelu(x) = x/2 (1 + erf(x / sqrt 2))
  __device__ __forceinline__ f32x4 operator()(f32x4 v) const {
#pragma unroll
    for (int i = 0; i < 4; i++) v[i] = 0.5f * v[i] * (1.0f + erff(v[i] * 0.70710678118654752f));
    return v;
  }
};
template <typename T, bool GELU> struct LinearPol {
  static constexpr bool A_KS = false, B_KS = true, SPLIT_K = false, ACC_T = true;
  static constexpr int EPI = GELU ? 2 : 1;
  static constexpr bool EPI_LDS = false;
  const T *In, *Wt;
  T *Out;
  int rows, K, N;
  __device__ __forceinline__ GemmCtx setup(int) const { return GemmCtx{rows, N, K, 0, 0, 0}; }
  __device__ __forceinline__ bool a_linear(int) const { return true; }
  __device__ __forceinline__ bool b_linear(int) const { return true; }
  __device__ __forceinline__ const T *a_ptr(const GemmCtx &, int m, int k) const { return In + (size_t)m * K + k; }
  __device__ __forceinline__ const T *b_ptr(const GemmCtx &, int n, int k) const { return Wt + (size_t)k * N + n; }
  template <int TM, int TN>
  __device__ __forceinline__ void epilogue(const GemmCtx &x, const WaveAccT<TM, TN> &acc, int m_w, int n_w,
                                           int lane, void *wave_lds) const {
    T *o = Out;
    const int N_ = N;
    auto row = [=](int m) { return o + (size_t)m * N_; };
    auto col = [](int n) { return n; };
    auto one = [](int) { return 1.0f; };
    if constexpr (GELU) store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N, row, col, one, ElemGelu());
    else store_rows<T, TM, TN>(acc, m_w, n_w, lane, x.M, x.N, row, col, one);
  }
};

// Probabilities (fp32 accumulator registers) -> B-operand fragment slots.
__device__ __forceinline__ void pack_probs(Frag<bf16_t> &f, const f32x4 &lo, const f32x4 &hi) {
  typedef float f32x8 __attribute__((ext_vector_type(8)));
  f32x8 all = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  f.v = __builtin_convertvector(all, bf16x8);  // four packed conversions
}
__device__ __forceinline__ void pack_probs(Frag<float> &f, const f32x4 &lo, const f32x4 &hi) {
#pragma unroll
  for (int r = 0; r < 4; r++) { f.v[r] = lo[r]; f.v[4 + r] = hi[r]; }
}

template <typename T, int DH>
__global__ __launch_bounds__(256) void k_attn(const T *__restrict__ Q, const T *__restrict__ Kx,
                                             const T *__restrict__ V, T *__restrict__ O, int Lq, int L, int H,
                                             float scale_log2, const float *__restrict__ Zs, int D, T *__restrict__ Oe) {
  constexpr int EPP = 16 / (int)sizeof(T);
  constexpr int LD = DH + EPP;        // LDS row stride (elements) of the K and V tiles [64][DH]
  constexpr int KK = DH / 32;         // fragments along head_dim
  constexpr int DT = DH / 16;         // output tiles along head_dim
  constexpr int QT = 2;               // query tiles (of 16) per wave
  constexpr int NP = 64 * DH / EPP / 256;
  __shared__ __align__(16) T Ks[64 * LD];
  __shared__ __align__(16) T Vs[64 * LD];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const int h = blockIdx.y, b = blockIdx.z;
  // Lq queries attend to L keys / values (the same tokens in self-attention)
  const size_t head = ((size_t)b * H + h) * L * DH;
  const T *Qh = Q + ((size_t)b * H + h) * Lq * DH, *Kh = Kx + head, *Vh = V + head;
  const int q_w = blockIdx.x * 128 + w * 32;

  // queries as B-operand fragments: lane = query column, slots = head_dim 32 kk + 8 g + i
  Frag<T> fq[QT][KK];
#pragma unroll
  for (int qt = 0; qt < QT; qt++) {
    int q = q_w + 16 * qt + c;
    q = q < Lq ? q : Lq - 1;
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      const T *src = Qh + (size_t)q * DH + 32 * kk + 8 * g;
      if constexpr (sizeof(T) == 2) {
        Pkt pk = pkt_load(src);
        fq[qt][kk] = __builtin_bit_cast(Frag<T>, pk);
      } else {
        Pkt p0 = pkt_load(src), p1 = pkt_load(src + 4);
        struct { Pkt a, b; } two = {p0, p1};
        fq[qt][kk] = __builtin_bit_cast(Frag<T>, two);
      }
    }
  }

  f32x4 oacc[DT][QT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int qt = 0; qt < QT; qt++) oacc[dt][qt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int qt = 0; qt < QT; qt++) { m_run[qt] = -__builtin_inff(); l_run[qt] = 0.f; }

  int lds_off[NP], g_row[NP], g_col[NP];
#pragma unroll
  for (int i = 0; i < NP; i++) {
    int q = tid + 256 * i;
    constexpr int PPR = DH / EPP;
    g_row[i] = q / PPR; g_col[i] = (q % PPR) * EPP;
    lds_off[i] = g_row[i] * LD + g_col[i];
  }

  Pkt rk[NP], rv[NP];
  auto fetch = [&](int key0) {
#pragma unroll
    for (int i = 0; i < NP; i++) {
      int key = key0 + g_row[i];
      key = key < L ? key : L - 1;  // rows past the end are masked below
      rk[i] = pkt_load(Kh + (size_t)key * DH + g_col[i]);
      rv[i] = pkt_load(Vh + (size_t)key * DH + g_col[i]);
    }
  };

  fetch(0);
  for (int key0 = 0; key0 < L; key0 += 64) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NP; i++) { pkt_store(Ks + lds_off[i], rk[i]); pkt_store(Vs + lds_off[i], rv[i]); }
    __syncthreads();
    if (key0 + 64 < L) fetch(key0 + 64);

    // transposed scores: st[kt][qt] holds keys 16 kt + 4 g + r (rows) of query c (column)
    f32x4 st[4][QT];
#pragma unroll
    for (int kt = 0; kt < 4; kt++)
#pragma unroll
      for (int qt = 0; qt < QT; qt++) st[kt][qt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; kk++)
#pragma unroll
      for (int kt = 0; kt < 4; kt++) {
        Frag<T> fk;
        frag_load_kc(fk, Ks + (16 * kt + c) * LD + 32 * kk + 8 * g);
#pragma unroll
        for (int qt = 0; qt < QT; qt++) mma16(st[kt][qt], fk, fq[qt][kk]);
      }

    const bool tail = key0 + 64 > L;
    Frag<T> fp[QT][2];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
      float mx = -__builtin_inff();
#pragma unroll
      for (int kt = 0; kt < 4; kt++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
          float sv = st[kt][qt][r] * scale_log2;
          if (tail && key0 + 16 * kt + 4 * g + r >= L) sv = -__builtin_inff();
          st[kt][qt][r] = sv;
          mx = fmaxf(mx, sv);
        }
      mx = fmaxf(mx, wave_xor_f32(mx, 16));
      mx = fmaxf(mx, wave_xor_f32(mx, 32));
      float m_new = fmaxf(m_run[qt], mx);
      float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
      m_run[qt] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; kt++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
          float pv = __builtin_amdgcn_exp2f(st[kt][qt][r] - m_new);
          st[kt][qt][r] = pv;
          psum += pv;
        }
      l_run[qt] = l_run[qt] * alpha + psum;
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int r = 0; r < 4; r++) oacc[dt][qt][r] *= alpha;
      pack_probs(fp[qt][0], st[0][qt], st[1][qt]);
      pack_probs(fp[qt][1], st[2][qt], st[3][qt]);
    }

    // O^T[dh][q] += sum_keys V[key][dh] P^T[key][q]; slot s of k-group g is key 32 u + 4 g + s
    // (s < 4) or 32 u + 16 + 4 g + s - 4, matching how the probabilities were packed.
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
      for (int dt = 0; dt < DT; dt++) {
        Frag<T> fv;
        frag_load_ks(fv, Vs, LD, 32 * u + 4 * g, 32 * u + 16 + 4 * g, 16 * dt, lane);
#pragma unroll
        for (int qt = 0; qt < QT; qt++) mma16(oacc[dt][qt], fv, fp[qt][u]);
      }
  }

  // O[b][q][h * DH + dh]: lane holds query c and head_dim rows 16 dt + 4 g + r
  const int Cw = H * DH;
#pragma unroll
  for (int qt = 0; qt < QT; qt++) {
    float l = l_run[qt];
    l += wave_xor_f32(l, 16);
    l += wave_xor_f32(l, 32);
    float inv = 1.0f / l;
    int q = q_w + 16 * qt + c;
    if (q >= Lq) continue;
    if (Zs && q < D) inv /= fmaxf(Zs[(size_t)b * D + q], 1e-20f);  // unmerge input: O / Z
    // (extra-token rows straight to their own output when the caller has one)
    T *dst = (Oe && q >= D ? Oe + ((size_t)b * (Lq - D) + (q - D)) * Cw : O + ((size_t)b * Lq + q) * Cw) + h * DH + 4 * g;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) {
      alignas(16) T o[4];
#pragma unroll
      for (int r = 0; r < 4; r++) o[r] = from_f32<T>(oacc[dt][qt][r] * inv);
      if (sizeof(T) == 2) *reinterpret_cast<u32x2 *>(dst + 16 * dt) = *reinterpret_cast<u32x2 *>(o);
      else *reinterpret_cast<u32x4 *>(dst + 16 * dt) = *reinterpret_cast<u32x4 *>(o);
    }
  }
}

// Maximum / sum over the four 16-lane rows of a wave without LDS traffic: the gfx950 row-swap
// instructions exchange odd with even rows (16) and the upper with the lower half (32); after each
// swap the two results hold the two partners of every lane.
// Maxima as single instructions: fmaxf() would first copy each operand through v_max(x, x) to
// quiet signalling NaNs, which scores never are.
__device__ __forceinline__ float max2_f32(float a, float b) {
  float d;
  asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
__device__ __forceinline__ float max3_f32(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}
__device__ __forceinline__ float rows4_max_f32(float v) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m = max2_f32(__builtin_bit_cast(float, (uint32_t)a[0]), __builtin_bit_cast(float, (uint32_t)a[1]));
  const uint32_t w = __builtin_bit_cast(uint32_t, m);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return max2_f32(__builtin_bit_cast(float, (uint32_t)b[0]), __builtin_bit_cast(float, (uint32_t)b[1]));
}
__device__ __forceinline__ float rows4_sum_f32(float v) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m = __builtin_bit_cast(float, (uint32_t)a[0]) + __builtin_bit_cast(float, (uint32_t)a[1]);
  const uint32_t w = __builtin_bit_cast(uint32_t, m);
  const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __builtin_bit_cast(float, (uint32_t)b[0]) + __builtin_bit_cast(float, (uint32_t)b[1]);
}

// The same attention with K and V tiles copied global -> LDS by the load-to-LDS path through a ring
// of four tiles (one barrier per 64 keys, two tiles of loads in flight) and bank-conflict-free
// swizzled tiles; the softmax scale is folded into the exponent's FMA.
// Software pipeline inside each wave: the score products of tile t + 1 are issued BEFORE the
// softmax of tile t, so that the matrix cores work on them while the vector ALU does the maxima,
// exponentials and packing of tile t (a wave executes in order; with one or two waves per SIMD
// nothing else would overlap the two).
// The number of waves per workgroup is the launch's choice (blockDim.x / 64, four to twelve), 16 QT
// queries each: with one query tile per wave it sets how many queries a workgroup takes and with
// that how evenly the grid fills the SIMDs (launch_attn picks it per shape).  Many waves with one
// tile each beat few waves with two: a wave alone overlaps its matrix and vector work poorly, and
// the ring of a 128-wide head leaves room for one workgroup per CU only.  The first four waves
// fetch the K / V tiles (the first eight where a row is 256 bytes or more: such launches have at
// least eight).
template <typename T, int DH, int QT>
__global__ __launch_bounds__(QT == 1 ? 768 : 256, QT == 1 ? (DH * sizeof(T) >= 256 ? 3 : 4) : (DH * sizeof(T) >= 256 ? 1 : 2)) void k_attn_async(
    const T *__restrict__ Q, const T *__restrict__ Kx, const T *__restrict__ V, T *__restrict__ O, int Lq, int L, int H,
    float scale_log2, const float *__restrict__ Zs, int D, T *__restrict__ Oe) {
  constexpr int ES = (int)sizeof(T), EPP = 16 / ES;
  constexpr int PPR = DH / EPP;       // 16-byte packets per K / V row
  constexpr int KK = DH / 32, DT = DH / 16, STAGES = 4;  // QT: query tiles (of 16) per wave
  constexpr int CH = PPR;             // 1 KiB chunks per 64-row tile
  constexpr int LW = QT == 1 && DH * ES >= 256 ? 8 : 4;  // waves that fetch the K / V tiles (the first LW)
  constexpr int NI = CH / LW;         // load instructions per loading wave per tile, for K and for V
  const int QB = (int)(blockDim.x >> 6) * 16 * QT;  // queries per workgroup
  constexpr int TILE = 64 * DH;
  __shared__ __align__(1024) T Ks[STAGES][TILE];
  __shared__ __align__(1024) T Vs[STAGES][TILE];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  // one-dimensional grid over (sample, head, query block), remapped so that the blocks an XCD
  // receives are neighbours: the query blocks of a head then share that head's K and V in one L2
  // (Lq queries attend to L keys / values: the same tokens in self-attention)
  const int nq = (Lq + QB - 1) / QB;
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  const int qb = work % nq, h = (work / nq) % H, b = work / (nq * H);
  const size_t head = ((size_t)b * H + h) * L * DH;
  const T *Qh = Q + ((size_t)b * H + h) * Lq * DH, *Kh = Kx + head, *Vh = V + head;
  const int q_w = qb * QB + w * (16 * QT);
  const int nt = (L + 63) / 64;

  Frag<T> fq[QT][KK];
#pragma unroll
  for (int qt = 0; qt < QT; qt++) {
    int q = q_w + 16 * qt + c;
    q = q < Lq ? q : Lq - 1;
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      const T *src = Qh + (size_t)q * DH + 32 * kk + 8 * g;
      if constexpr (sizeof(T) == 2) {
        Pkt pk = pkt_load(src);
        fq[qt][kk] = __builtin_bit_cast(Frag<T>, pk);
      } else {
        Pkt p0 = pkt_load(src), p1 = pkt_load(src + 4);
        struct { Pkt a, b; } two = {p0, p1};
        fq[qt][kk] = __builtin_bit_cast(Frag<T>, two);
      }
    }
  }

  // what this lane fetches for its chunks: tile row and element offset inside the row
  // (element offsets from the head's first row: the tile's base stays in scalar registers)
  int k_row[NI], k_off[NI], v_off[NI];
  const bool loader = w < LW;
  const int wl = w & (LW - 1);
#pragma unroll
  for (int t = 0; t < NI; t++) {
    const int ch = wl * NI + t, row = ch * (64 / PPR) + lane / PPR, pos = lane % PPR;
    k_row[t] = row;
    k_off[t] = row * DH + ((pos & ~7) | ((pos ^ row) & 7)) * EPP;
    v_off[t] = row * DH + SwzTile<T>::template ks_slot<PPR, true>(row, pos) * EPP;
  }
  // LDS byte addresses of this wave's first chunk in stage 0 (scalar registers)
  const uint32_t ks_addr = lds_addr_of(&Ks[0][0]) + (uint32_t)__builtin_amdgcn_readfirstlane(wl) * (NI * 1024);
  const uint32_t vs_addr = lds_addr_of(&Vs[0][0]) + (uint32_t)__builtin_amdgcn_readfirstlane(wl) * (NI * 1024);
  // (the tile's base address is wave-uniform and the lanes' offsets inside a tile never change: the
  // loads take the base from scalar registers and cost no vector instruction for their addresses)
  uint32_t k_offb[NI], v_offb[NI];
#pragma unroll
  for (int t = 0; t < NI; t++) { k_offb[t] = (uint32_t)k_off[t] * ES; v_offb[t] = (uint32_t)v_off[t] * ES; }
  auto issue = [&](int st, int it) {
    if (!loader) return;  // (a wave without loads passes every vmcnt wait below at once)
    const ptrdiff_t adv = (ptrdiff_t)it * 64 * DH;
    if ((it + 1) * 64 <= L) {  // uniform: only the last tile can reach past the end
      const T *kb = Kh + adv, *vb = Vh + adv;
#pragma unroll
      for (int t = 0; t < NI; t++) {
        load_to_lds16_from(kb, k_offb[t], ks_addr + (uint32_t)(st * TILE * ES + t * 1024));
        load_to_lds16_from(vb, v_offb[t], vs_addr + (uint32_t)(st * TILE * ES + t * 1024));
      }
    } else {  // rows past the end repeat row L - 1 and are masked below
#pragma unroll
      for (int t = 0; t < NI; t++) {
        const ptrdiff_t a = it * 64 + k_row[t] >= L ? (ptrdiff_t)(L - 1 - k_row[t]) * DH : adv;
        load_to_lds16_at(Kh + (a + k_off[t]), ks_addr + (uint32_t)(st * TILE * ES + t * 1024));
        load_to_lds16_at(Vh + (a + v_off[t]), vs_addr + (uint32_t)(st * TILE * ES + t * 1024));
      }
    }
  };

  f32x4 oacc[DT][QT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int qt = 0; qt < QT; qt++) oacc[dt][qt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run[QT], l_run[QT];  // reference point (a recent maximum of the raw scores) and sum per query
  constexpr float kSlackLog2 = 8.0f;
  const float slack = kSlackLog2 / scale_log2;  // in units of the raw scores
#pragma unroll
  for (int qt = 0; qt < QT; qt++) { m_run[qt] = -__builtin_inff(); l_run[qt] = 0.f; }

  // transposed scores of one tile: st[kt][qt] holds keys 16 kt + 4 g + r (rows) of query c (column)
  // All K fragments of the tile are requested before the first product (a scheduling fence keeps
  // the compiler from folding each read back in front of its use: it would wait out the LDS
  // latency once per fragment instead of once per tile).
  // (in batches of KB k-groups: all at once where the registers allow)
  auto scores = [&](f32x4 (&st)[4][QT], const T *kt_) {
    constexpr int KB = (QT == 1 && KK > 2) ? 2 : KK;
#pragma unroll
    for (int k0 = 0; k0 < KK; k0 += KB) {
      Frag<T> fk[KB][4];
#pragma unroll
      for (int kk = 0; kk < KB; kk++)
#pragma unroll
        for (int kt = 0; kt < 4; kt++) frag_load_kcw_sw<PPR>(fk[kk][kt], kt_, 16 * kt + c, 32 * (k0 + kk) + 8 * g);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < KB; kk++)
#pragma unroll
        for (int kt = 0; kt < 4; kt++)
#pragma unroll
          for (int qt = 0; qt < QT; qt++) {
            if (k0 + kk == 0) st[kt][qt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            mma16(st[kt][qt], fk[kk][kt], fq[qt][k0 + kk]);
          }
      if (k0 + KB < KK) __builtin_amdgcn_sched_barrier(0);
    }
  };
  // online softmax of one tile's scores and O^T += V^T P^T
  auto softmax_pv = [&](f32x4 (&st)[4][QT], const T *vt_, int key0) {
    if (key0 + 64 > L) {  // only the last tile can reach past the end (uniform branch)
#pragma unroll
      for (int qt = 0; qt < QT; qt++)
#pragma unroll
        for (int kt = 0; kt < 4; kt++)
#pragma unroll
          for (int r = 0; r < 4; r++)
            if (key0 + 16 * kt + 4 * g + r >= L) st[kt][qt][r] = -__builtin_inff();
    }
    Frag<T> fp[QT][2];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
      float mx = max3_f32(st[0][qt][0], st[0][qt][1], st[0][qt][2]);
      mx = max3_f32(mx, st[0][qt][3], st[1][qt][0]);
#pragma unroll
      for (int kt = 1; kt < 4; kt++) {
        mx = max3_f32(mx, st[kt][qt][1], st[kt][qt][2]);
        if (kt < 3) mx = max3_f32(mx, st[kt][qt][3], st[kt + 1][qt][0]);
        else mx = max2_f32(mx, st[kt][qt][3]);
      }
      mx = rows4_max_f32(mx);
      // The reference point of the exponentials follows the running maximum lazily: it moves (and
      // the sums so far are rescaled) only when some row's maximum has grown by more than
      // kSlackLog2 in the exponent, i.e. almost never after the first tile.  Until then the
      // exponentials are at most 2^kSlackLog2, and the final O / l does not depend on the
      // reference point.
      const bool grew = __any(mx > m_run[qt] + slack);
      if (grew) {
        const float m_new = fmaxf(m_run[qt], mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run[qt] - m_new) * scale_log2);
        m_run[qt] = m_new;
        l_run[qt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
#pragma unroll
          for (int r = 0; r < 4; r++) oacc[dt][qt][r] *= alpha;
      }
      const float mc = m_run[qt] * scale_log2;
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; kt++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
          float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][qt][r], scale_log2, -mc));
          st[kt][qt][r] = pv;
          psum += pv;
        }
      l_run[qt] += psum;
      pack_probs(fp[qt][0], st[0][qt], st[1][qt]);
      pack_probs(fp[qt][1], st[2][qt], st[3][qt]);
    }
    // slot s of k-group g is key 32 u + 4 g + s (s < 4) or 32 u + 16 + 4 g + s - 4, matching how
    // the probabilities were packed
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
      for (int dt = 0; dt < DT; dt++) {
        Frag<T> fv;
        frag_load_ks_sw<PPR, true>(fv, vt_, 32 * u + 4 * g, 32 * u + 16 + 4 * g, 16 * dt, lane);
#pragma unroll
        for (int qt = 0; qt < QT; qt++) mma16(oacc[dt][qt], fv, fp[qt][u]);
      }
  };

  // the query loads must have landed before the ring starts: from here on only the ring's own
  // loads are outstanding, and only the waits below order them
  wait_vmcnt<0>();
  issue(0, 0);
  if (nt > 1) issue(1, 1);
  if (nt > 2) issue(2, 2);
  if (nt > 2) wait_vmcnt<4 * NI>(); else if (nt > 1) wait_vmcnt<2 * NI>(); else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  f32x4 sa[4][QT], sb[4][QT];
  scores(sa, Ks[0]);
  // one step per 64 keys; ring position and score buffer are compile-time constants of each of
  // the four unrolled copies
  auto tile_step = [&](auto stage_c, f32x4 (&cur)[4][QT], f32x4 (&nxt)[4][QT], int it) {
    constexpr int ST = decltype(stage_c)::value;
    if (it + 1 < nt) {
      // this wave's part of tile it + 1 has landed (tile it + 2 may still be in flight); after the
      // barrier so has everyone's, and every wave is done with tile it - 1
      if (it + 2 < nt) wait_vmcnt<2 * NI>(); else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      if (it + 3 < nt) issue((ST + 3) % STAGES, it + 3);
      scores(nxt, Ks[(ST + 1) % STAGES]);
      __builtin_amdgcn_sched_barrier(0);
    }
    softmax_pv(cur, Vs[ST], it * 64);
  };
  for (int it = 0; it < nt; it += 4) {
    tile_step(std::integral_constant<int, 0>{}, sa, sb, it);
    if (it + 1 < nt) tile_step(std::integral_constant<int, 1>{}, sb, sa, it + 1);
    if (it + 2 < nt) tile_step(std::integral_constant<int, 2>{}, sa, sb, it + 2);
    if (it + 3 < nt) tile_step(std::integral_constant<int, 3>{}, sb, sa, it + 3);
  }

  const int Cw = H * DH;
#pragma unroll
  for (int qt = 0; qt < QT; qt++) {
    const float l = rows4_sum_f32(l_run[qt]);
    float inv = 1.0f / l;
    int q = q_w + 16 * qt + c;
    if (q >= Lq) continue;
    if (Zs && q < D) inv /= fmaxf(Zs[(size_t)b * D + q], 1e-20f);  // unmerge input: O / Z
    // (extra-token rows straight to their own output when the caller has one)
    T *dst = (Oe && q >= D ? Oe + ((size_t)b * (Lq - D) + (q - D)) * Cw : O + ((size_t)b * Lq + q) * Cw) + h * DH + 4 * g;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) {
      alignas(16) T o[4];
#pragma unroll
      for (int r = 0; r < 4; r++) o[r] = from_f32<T>(oacc[dt][qt][r] * inv);
      if (sizeof(T) == 2) *reinterpret_cast<u32x2 *>(dst + 16 * dt) = *reinterpret_cast<u32x2 *>(o);
      else *reinterpret_cast<u32x4 *>(dst + 16 * dt) = *reinterpret_cast<u32x4 *>(o);
    }
  }
}

// Waves per workgroup for k_attn_async with one query tile per wave.  Model (fitted to sweeps of
// the wave count over sequence lengths 512 .. 8192): workgroups are placed `cap` to a CU (LDS ring
// and register file) in rounds over the 256 CUs; the busiest SIMD of a CU then holds
// k = cap * ceil(nw / 4) waves (a second workgroup lands on the SIMDs like the first), and a round
// costs max(kAlone, k) units per key tile: several waves on a SIMD are bound by their vector-ALU
// work, one or two by their own dependent chain (kAlone: about 2 for rows under 256 bytes, 2.3
// above).  The choice with the least total wins; how ties go is said in the function.
static int attn_waves(int L, int heads_x_batch, int ring_bytes, int waves_per_cu, int min_waves, float kAlone) {
  float cost[13];
  long wgs_of[13];
  float least = 0.f;
  for (int nw = min_waves; nw <= 12; nw++) {
    cost[nw] = -1.f;
    const int cap = std::min((160 * 1024) / ring_bytes, waves_per_cu / nw);
    if (cap < 1) continue;
    const long wgs = (long)((L + 16 * nw - 1) / (16 * nw)) * heads_x_batch;
    const long slots = 256L * cap, full = wgs / slots, rem = wgs % slots;
    const int per_simd = (nw + 3) / 4;
    float c = (float)full * std::max(kAlone, (float)(cap * per_simd));
    if (rem) c += std::max(kAlone, (float)((int)((rem + 255) / 256) * per_simd));
    cost[nw] = c;
    wgs_of[nw] = wgs;
    if (least == 0.f || c < least) least = c;
  }
  // among the choices within 3% of the least: the one that spreads one workgroup per CU over the
  // most CUs (measured 5-8% ahead of its equals), else eight waves, else the first
  int best = -1;
  for (int nw = min_waves; nw <= 12; nw++) {
    if (cost[nw] < 0.f || cost[nw] > least * 1.03f) continue;
    if (wgs_of[nw] <= 256 && (best < 0 || wgs_of[best] > 256 || wgs_of[nw] > wgs_of[best])) best = nw;
    else if (best < 0 || (nw == 8 && wgs_of[best] > 256)) best = nw;
  }
  return best < 0 ? 8 : best;
}

#ifndef TOMA_ATTN_QT
#define TOMA_ATTN_QT 1   // query tiles per wave: 1 (any number of waves) or 2 (four waves)
#endif
// nw: waves per workgroup, 0 = chosen by attn_waves
template <typename T, int DH>
static void launch_attn(const Shape &s, int Lq, int Lk, const T *Q, const T *K, const T *V, T *O, const float *Zs,
                        T *Oe, hipStream_t st, int nw = 0) {
  float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  KernelTimer kt(K_ATTN, st);
  // load-to-LDS pipeline when a row is at least eight packets and the ring of four tiles fits the LDS
  constexpr int kRowPackets = DH * (int)sizeof(T) / 16;
  constexpr int kRing = 4 * 2 * 64 * DH * (int)sizeof(T);
  if constexpr (kRowPackets >= 8 && kRing <= 160 * 1024 - 4096) {
    if (TOMA_ATTN_QT == 1) {
      constexpr bool kWide = DH * sizeof(T) >= 256;  // three waves per SIMD fit the registers, else four
      if (nw < (kWide ? 8 : 4) || nw > 12) nw = attn_waves(Lq, s.heads * s.B, kRing, kWide ? 12 : 16, kWide ? 8 : 4, kWide ? 2.3f : 2.0f);
      dim3 grid((Lq + 16 * nw - 1) / (16 * nw) * s.heads * s.B);
      hipLaunchKernelGGL((k_attn_async<T, DH, 1>), grid, dim3(64 * nw), 0, st, Q, K, V, O, Lq, Lk, s.heads, scale_log2, Zs, s.D, Oe);
    } else {
      dim3 grid((Lq + 127) / 128 * s.heads * s.B);
      hipLaunchKernelGGL((k_attn_async<T, DH, 2>), grid, dim3(256), 0, st, Q, K, V, O, Lq, Lk, s.heads, scale_log2, Zs, s.D, Oe);
    }
    return;
  }
  dim3 grid((Lq + 127) / 128, s.heads, s.B);
  hipLaunchKernelGGL((k_attn<T, DH>), grid, dim3(256), 0, st, Q, K, V, O, Lq, Lk, s.heads, scale_log2, Zs, s.D, Oe);
}

template <typename T>
static int attend_typed(const Shape &s, const void *Xm, const void *Xe, const void *Wq, const void *Wk,
                        const void *Wv, const void *Wo, void *O, const float *Zs, void *O_extra, char *ws,
                        const Workspace &w, hipStream_t st) {
  T *Q = reinterpret_cast<T *>(ws + w.q), *K = reinterpret_cast<T *>(ws + w.k), *V = reinterpret_cast<T *>(ws + w.v);
  T *Oe = static_cast<T *>(O_extra);
  QkvPol<T> p{};
  p.Xm = static_cast<const T *>(Xm); p.Xe = static_cast<const T *>(Xe);
  p.W[0] = static_cast<const T *>(Wq); p.W[1] = static_cast<const T *>(Wk); p.W[2] = static_cast<const T *>(Wv);
  p.out[0] = Q; p.out[1] = K; p.out[2] = V;
  p.B = s.B; p.D = s.D; p.Tx = s.T; p.L = s.L; p.C = s.C; p.H = s.heads; p.dh = s.head_dim; p.Kin = s.C;
  p.dh_sh = -1;
  for (int sh = 0; sh < 16; sh++) if ((1 << sh) == s.head_dim) p.dh_sh = sh;
  launch_gemm<T>(K_QKV, p, s.B * s.L, s.C, s.C, 3, st);
  T *Oh = Wo ? reinterpret_cast<T *>(ws + w.oh) : static_cast<T *>(O);
  switch (s.head_dim) {
    case 32: launch_attn<T, 32>(s, s.L, s.L, Q, K, V, Oh, Wo ? nullptr : Zs, Wo ? nullptr : Oe, st); break;
    case 64: launch_attn<T, 64>(s, s.L, s.L, Q, K, V, Oh, Wo ? nullptr : Zs, Wo ? nullptr : Oe, st); break;
    case 128: launch_attn<T, 128>(s, s.L, s.L, Q, K, V, Oh, Wo ? nullptr : Zs, Wo ? nullptr : Oe, st); break;
    default: return TOMA_ERR_UNSUPPORTED;
  }
  if (Wo) {
    ProjPol<T> pp{};
    pp.In = Oh; pp.Wt = static_cast<const T *>(Wo); pp.Out = static_cast<T *>(O);
    pp.rows = s.B * s.L; pp.C = s.C; pp.L = s.L; pp.D = s.D; pp.Zs = Zs; pp.Oe = Oe;
    launch_gemm<T>(K_PROJ, pp, s.B * s.L, s.C, s.C, 1, st);
  }
  return launch_status();
}

int launch_attend(const Shape &s, const void *Xm, const void *Xe, const void *Wq, const void *Wk,
                  const void *Wv, const void *Wo, void *O, const float *Zs, void *O_extra, char *ws,
                  const Workspace &w, hipStream_t st) {
  return s.dtype == TOMA_BF16 ? attend_typed<bf16_t>(s, Xm, Xe, Wq, Wk, Wv, Wo, O, Zs, O_extra, ws, w, st)
                              : attend_typed<float>(s, Xm, Xe, Wq, Wk, Wv, Wo, O, Zs, O_extra, ws, w, st);
}

// Cross-attention: queries from the L rows of U, keys / values from t_ctx context rows of width c_ctx.
template <typename T>
static int cross_typed(const Shape &s, const void *U, const void *Ctx, int t_ctx, int c_ctx, const void *Wq,
                       const void *Wk, const void *Wv, const void *Wo, void *O, char *ws, const Workspace &w,
                       hipStream_t st) {
  T *Q = reinterpret_cast<T *>(ws + w.q), *K = reinterpret_cast<T *>(ws + w.k), *V = reinterpret_cast<T *>(ws + w.v);
  QkvPol<T> pq{};
  pq.Xm = static_cast<const T *>(U); pq.Xe = nullptr;
  pq.W[0] = static_cast<const T *>(Wq); pq.W[1] = pq.W[2] = nullptr;
  pq.out[0] = Q; pq.out[1] = pq.out[2] = nullptr;
  pq.B = s.B; pq.D = s.L; pq.Tx = 0; pq.L = s.L; pq.C = s.C; pq.H = s.heads; pq.dh = s.head_dim; pq.Kin = s.C;
  pq.dh_sh = -1;
  for (int sh = 0; sh < 16; sh++) if ((1 << sh) == s.head_dim) pq.dh_sh = sh;
  launch_gemm<T>(K_QKV, pq, s.B * s.L, s.C, s.C, 1, st);
  QkvPol<T> pk = pq;
  pk.Xm = static_cast<const T *>(Ctx);
  pk.W[0] = static_cast<const T *>(Wk); pk.W[1] = static_cast<const T *>(Wv);
  pk.out[0] = K; pk.out[1] = V;
  pk.D = t_ctx; pk.L = t_ctx; pk.Kin = c_ctx;
  launch_gemm<T>(K_QKV, pk, s.B * t_ctx, s.C, c_ctx, 2, st);
  T *Oh = Wo ? reinterpret_cast<T *>(ws + w.oh) : static_cast<T *>(O);
  switch (s.head_dim) {
    case 32: launch_attn<T, 32>(s, s.L, t_ctx, Q, K, V, Oh, nullptr, nullptr, st); break;
    case 64: launch_attn<T, 64>(s, s.L, t_ctx, Q, K, V, Oh, nullptr, nullptr, st); break;
    case 128: launch_attn<T, 128>(s, s.L, t_ctx, Q, K, V, Oh, nullptr, nullptr, st); break;
    default: return TOMA_ERR_UNSUPPORTED;
  }
  if (Wo) {
    ProjPol<T> pp{};
    pp.In = Oh; pp.Wt = static_cast<const T *>(Wo); pp.Out = static_cast<T *>(O);
    pp.rows = s.B * s.L; pp.C = s.C; pp.L = s.L; pp.D = s.D; pp.Zs = nullptr; pp.Oe = nullptr;
    launch_gemm<T>(K_PROJ, pp, s.B * s.L, s.C, s.C, 1, st);
  }
  return launch_status();
}

int launch_cross_attend(const Shape &s, const void *U, const void *Ctx, int t_ctx, int c_ctx, const void *Wq,
                        const void *Wk, const void *Wv, const void *Wo, void *O, char *ws, const Workspace &w,
                        hipStream_t st) {
  return s.dtype == TOMA_BF16 ? cross_typed<bf16_t>(s, U, Ctx, t_ctx, c_ctx, Wq, Wk, Wv, Wo, O, ws, w, st)
                              : cross_typed<float>(s, U, Ctx, t_ctx, c_ctx, Wq, Wk, Wv, Wo, O, ws, w, st);
}

template <typename T>
static int mlp_typed(int rows, int C, int hidden, const void *In, const void *W1, const void *W2, void *Hbuf, void *Out,
                     hipStream_t st) {
  LinearPol<T, true> up{};
  up.In = static_cast<const T *>(In); up.Wt = static_cast<const T *>(W1); up.Out = static_cast<T *>(Hbuf);
  up.rows = rows; up.K = C; up.N = hidden;
  launch_gemm<T>(K_MLP_UP, up, rows, hidden, C, 1, st);
  LinearPol<T, false> down{};
  down.In = static_cast<const T *>(Hbuf); down.Wt = static_cast<const T *>(W2); down.Out = static_cast<T *>(Out);
  down.rows = rows; down.K = hidden; down.N = C;
  launch_gemm<T>(K_MLP_DOWN, down, rows, C, hidden, 1, st);
  return launch_status();
}

int launch_mlp(int dtype, int rows, int C, int hidden, const void *In, const void *W1, const void *W2, void *Hbuf,
               void *Out, hipStream_t st) {
  return dtype == TOMA_BF16 ? mlp_typed<bf16_t>(rows, C, hidden, In, W1, W2, Hbuf, Out, st)
                            : mlp_typed<float>(rows, C, hidden, In, W1, W2, Hbuf, Out, st);
}

}  // namespace toma
