// fp64 sums of squares of token rows and their reduction across the lanes of a row, shared by the
// block-score sweep and the prefill token-score sweep (Alg. 1: S_i = ||V_i||_2 / ||K_i||_2).
#pragma once

#include "pe_device.h"

namespace pe {

// acc + sum of squares of the elements of one 16-byte vector, in element order.
template <typename T>
__device__ __forceinline__ double sumsq_vec(const uint4& v, double acc) {
#pragma unroll
  for (int e = 0; e < Elem<T>::kPerVec; ++e) {
    const double x = (double)vec_elem<T>(v, e);
    acc = fma(x, x, acc);
  }
  return acc;
}

// Reduce-scatter of NV per-lane values over aligned groups of NV lanes: the result on lane l is the
// group total of value index bit_reverse(l & (NV-1)).
template <int NV, int STAGE_M = 1>
__device__ __forceinline__ double reduce_scatter_f64(double (&v)[NV], int lane) {
  if constexpr (NV == 1) {
    return v[0];
  } else {
    const bool up = (lane & STAGE_M) != 0;
    double w[NV / 2];
#pragma unroll
    for (int i = 0; i < NV / 2; ++i) {
      const double keep = up ? v[i + NV / 2] : v[i];
      const double send = up ? v[i] : v[i + NV / 2];
      w[i] = keep + lane_xor_f64<STAGE_M>(send);
    }
    return reduce_scatter_f64<NV / 2, STAGE_M * 2>(w, lane);
  }
}

// Sum over lane bits FROM, 2*FROM, ... < TO (every lane of the group gets the total).
template <int FROM, int TO>
__device__ __forceinline__ double all_reduce_f64(double v) {
  if constexpr (FROM >= TO) {
    return v;
  } else {
    return all_reduce_f64<FROM * 2, TO>(v + lane_xor_f64<FROM>(v));
  }
}

// From per-lane partial sums part[kv * NL + i] (kv: 0 = K, 1 = V; i = wave-load) to the token ratio:
// afterwards every lane holds ||V||/||K|| of token row i = bit_reverse((lane >> 1) & (NL-1)) of its
// lane group (lanes with equal (lane >> 1) & (NL-1) hold copies).  ||V|| = 0 gives 0, else ||K|| = 0
// gives +inf.
template <int NL, int LPR>
__device__ __forceinline__ double token_ratio_from_partials(double (&part)[2 * NL], int lane) {
  static_assert(2 * NL <= LPR, "needs at least as many lanes per row as partial sums");
  double tot = reduce_scatter_f64<2 * NL>(part, lane);
  tot = all_reduce_f64<2 * NL, LPR>(tot);
  const double nrm = sqrt(tot);
  const double other = lane_xor_f64<1>(nrm);
  const double nk = (lane & 1) ? other : nrm;
  const double nv = (lane & 1) ? nrm : other;
  double ratio = nv / nk;  // nk == 0 with nv > 0 is +inf by IEEE division
  if (nv == 0.0) ratio = 0.0;
  return ratio;
}

}  // namespace pe
