// Addressing of one merge region's tokens: which grid token is source s of merge region rho.
#pragma once
#include "toma_common.h"
#include "toma_internal.h"

namespace toma {

template <typename T> struct RegionView {
  const T *X;
  RegionMap map;
  int N, C, D, R, Nr, Dr;
  // Sources are enumerated region by region in both merge modes (local order inside a region), so
  // that the columns of A that a region's destinations actually weigh - its own tokens and a few
  // neighbours - are contiguous: with one merge region per sample, source s is token s % N_loc of
  // selection region s / N_loc.
  int sh_nloc, sh_tw, sh_pw;  // log2 of N_loc, tile_w and regions per grid row when all are powers of two, else -1
  __device__ __forceinline__ int token(int rho, int s) const {
    if (R != 1) return map.token(rho, s);
    if (sh_nloc >= 0) {  // the usual shapes: no divisions
      const int p = s >> sh_nloc, l = s & ((1 << sh_nloc) - 1);
      const int r = (p >> sh_pw) * map.tile_h + (l >> sh_tw), c = ((p & (map.pw - 1)) << sh_tw) + (l & (map.tile_w - 1));
      return r * map.W + c;
    }
    const int n_loc = map.tile_h * map.tile_w;
    return map.token(s / n_loc, s % n_loc);
  }
  // token(rho, s + step) - token(rho, s) does not depend on s (inside one selection region)
  __device__ __forceinline__ bool token_linear(int step) const {
    if (R == 1) return map.tile_w == map.W;  // full-width regions: region order is grid order
    return step % map.tile_w == 0;
  }
  // token(rho, s + i) - token(rho, s) does not depend on s for s a multiple of step and i < step:
  // steps start on a region row and stay inside one selection region
  __device__ __forceinline__ bool token_step_uniform(int step) const {
    return step % map.tile_w == 0 && (map.tile_h * map.tile_w) % step == 0;
  }
};

template <typename T> inline RegionView<T> make_view(const Shape &s, const void *X) {
  RegionView<T> v;
  v.X = static_cast<const T *>(X);
  v.map = RegionMap{s.W, s.tile_h, s.tile_w, s.W / s.tile_w};
  v.N = s.N; v.C = s.C; v.D = s.D; v.R = s.R; v.Nr = s.Nr; v.Dr = s.Dr;
  auto log2_exact = [](int x) { int sh = 0; while ((1 << sh) < x) sh++; return (1 << sh) == x ? sh : -1; };
  v.sh_nloc = log2_exact(s.n_loc); v.sh_tw = log2_exact(s.tile_w); v.sh_pw = log2_exact(v.map.pw);
  if (v.sh_nloc < 0 || v.sh_tw < 0 || v.sh_pw < 0) v.sh_nloc = v.sh_tw = v.sh_pw = -1;
  return v;
}

}  // namespace toma
