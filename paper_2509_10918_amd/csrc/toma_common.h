// Device-side building blocks shared by the ToMA kernels (gfx950 / CDNA4 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace toma {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// Token n of local position l in region p (tile-shaped regions; a stripe is tile_w == W).
struct RegionMap {
  int W, tile_h, tile_w, pw;  // pw = regions per grid row
  __device__ __forceinline__ int token(int p, int l) const {
    int r = (p / pw) * tile_h + l / tile_w;
    int c = (p % pw) * tile_w + l % tile_w;
    return r * W + c;
  }
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

// ---------------------------------------------------------------------------------------------
// MFMA fragments.  A fragment is what one lane feeds to a 16 x 16 x 32 product: lane l owns the
// matrix row (A operand) or column (B operand) l % 16 and eight k-slots of k-group l / 16.  With
// bf16 the eight slots are one v_mfma_f32_16x16x32_bf16 operand; with fp32 they are fed one slot
// at a time to eight v_mfma_f32_16x16x4_f32 (slot i of the four k-groups forms its K = 4).  The
// accumulator tile is the same for both: lane l holds column l % 16, rows 4 * (l / 16) + r.
// Which k value a slot stands for is the caller's choice, as long as A and B agree.
// ---------------------------------------------------------------------------------------------
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { bf16x8 v; };
template <> struct Frag<float> { float v[8]; };

__device__ __forceinline__ void mma16(f32x4 &acc, const Frag<bf16_t> &a, const Frag<bf16_t> &b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma16(f32x4 &acc, const Frag<float> &a, const Frag<float> &b) {
#pragma unroll
  for (int i = 0; i < 8; i++) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[i], b.v[i], acc, 0, 0, 0);
}

template <typename T> __device__ __forceinline__ void frag_zero(Frag<T> &f);
template <> __device__ __forceinline__ void frag_zero<bf16_t>(Frag<bf16_t> &f) {
#pragma unroll
  for (int i = 0; i < 8; i++) f.v[i] = (bf16_t)0.0f;
}
template <> __device__ __forceinline__ void frag_zero<float>(Frag<float> &f) {
#pragma unroll
  for (int i = 0; i < 8; i++) f.v[i] = 0.0f;
}

// Eight consecutive k of one row of a k-contiguous LDS tile.  p points at the first of them.
__device__ __forceinline__ void frag_load_kc(Frag<bf16_t> &f, const bf16_t *p) {
  f.v = *reinterpret_cast<const bf16x8 *>(p);
}
__device__ __forceinline__ void frag_load_kc(Frag<float> &f, const float *p) {
  f32x4 a = *reinterpret_cast<const f32x4 *>(p);
  f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; i++) { f.v[i] = a[i]; f.v[4 + i] = b[i]; }
}

// Fragment from a k-major LDS tile T[k][n] (n contiguous, row stride ld elements): slots 0..3 are
// k = ka..ka+3 and slots 4..7 are k = kb..kb+3, all for column nb + (lane % 16).
// bf16 uses the LDS transpose read: within 16 lanes, the lane j supplies the address of
// T[k0 + j / 4][nb + 4 * (j % 4)] (four n-contiguous values) and lane i receives T[k0 .. k0+3][nb + i].
__device__ __forceinline__ void frag_load_ks(Frag<bf16_t> &f, const bf16_t *tile, int ld, int ka, int kb,
                                             int nb, int lane) {
  typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;
  int j = lane & 15;
  const bf16_t *pa = tile + (ka + (j >> 2)) * ld + nb + 4 * (j & 3);
  const bf16_t *pb = tile + (kb + (j >> 2)) * ld + nb + 4 * (j & 3);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(pa));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(pb));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  f.v = __builtin_bit_cast(bf16x8, both);
}
__device__ __forceinline__ void frag_load_ks(Frag<float> &f, const float *tile, int ld, int ka, int kb,
                                             int nb, int lane) {
  int j = lane & 15;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    f.v[i] = tile[(ka + i) * ld + nb + j];
    f.v[4 + i] = tile[(kb + i) * ld + nb + j];
  }
}

// 16-byte global <-> register packets.
struct Pkt { u32x4 v; };
__device__ __forceinline__ Pkt pkt_load(const void *p) {
  Pkt r; r.v = *reinterpret_cast<const u32x4 *>(p); return r;
}
__device__ __forceinline__ Pkt pkt_zero() { Pkt r; r.v = (u32x4){0u, 0u, 0u, 0u}; return r; }
__device__ __forceinline__ void pkt_store(void *p, const Pkt &r) { *reinterpret_cast<u32x4 *>(p) = r.v; }

// Reductions inside each row of 16 lanes with DPP-modified instructions (no LDS traffic): after
// the call every lane of a 16-lane row holds the row's result.
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max_f32(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));   // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_f32<0x4E>(v));   // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp_f32<0x124>(v));  // row_ror 4
  v = fmaxf(v, dpp_f32<0x128>(v));  // row_ror 8
  return v;
}
__device__ __forceinline__ float row16_sum_f32(float v) {
  v += dpp_f32<0xB1>(v);
  v += dpp_f32<0x4E>(v);
  v += dpp_f32<0x124>(v);
  v += dpp_f32<0x128>(v);
  return v;
}

// Linear workgroup id -> tile id such that the ids an XCD receives (id mod 8) form a contiguous
// run of tiles.
__device__ __forceinline__ int xcd_remap(int id, int total) {
  const int per = total >> 3, body = per << 3;
  return id < body ? (id & 7) * per + (id >> 3) : id;
}

// Wave-level helpers (64 lanes).
__device__ __forceinline__ float wave_xor_f32(float v, int mask) { return __shfl_xor(v, mask, 64); }
__device__ __forceinline__ double wave_xor_f64(double v, int mask) { return __shfl_xor(v, mask, 64); }

}  // namespace toma
