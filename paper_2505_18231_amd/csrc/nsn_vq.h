// Nearest-codeword search (Eq. 1 with squared Euclidean distance) for one sub-vector per lane.
//
// Fast pass: fp32 expanded form ||c||^2 - 2 y.c over all 256 codewords, tracking the best
// two values.  If the runner-up is within a rounding-error window of the best, the decision
// is retaken in fp64 with the direct form sum (y_i - c_i)^2, lowest index on ties, so the
// chosen index equals an fp64 exhaustive search.
#pragma once

#include "nsn_device.h"

namespace nsn {

template <int SUB>
struct VqTables {
  double cx[kCodes][SUB];    // exact codeword values
  float neg2c[kCodes][SUB];  // -2 c rounded to fp32
  float cn[kCodes];          // ||c||^2 in fp32
  float cmax;                // max_c ||c||
};

// Fill the tables from fp64 codewords (all threads of the block take part; ends with a barrier).
template <int SUB, typename Load>
__device__ inline void vq_tables_fill(VqTables<SUB>& T, Load load_codeword_elem) {
  for (int c = threadIdx.x; c < kCodes; c += blockDim.x) {
    float n2 = 0.f;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      const double v = load_codeword_elem(c, i);
      T.cx[c][i] = v;
      const float f = (float)v;
      T.neg2c[c][i] = -2.f * f;
      n2 = fmaf(f, f, n2);
    }
    T.cn[c] = n2;
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    float m = 0.f;
    for (int c = threadIdx.x; c < kCodes; c += 64) m = fmaxf(m, T.cn[c]);
    m = wave_max(m);
    if (threadIdx.x == 0) T.cmax = sqrtf(m);
  }
  __syncthreads();
}

template <int SUB>
__device__ inline double exact_dist(const VqTables<SUB>& T, const double (&y)[SUB], int c) {
  double d = 0.0;
#pragma unroll
  for (int i = 0; i < SUB; ++i) {
    const double t = y[i] - T.cx[c][i];
    d = __dadd_rn(d, __dmul_rn(t, t));  // no fused contraction: plain sum of squares
  }
  return d;
}

// fp64 exhaustive search, direct form, lowest index on ties (the rare path of both searches)
template <int SUB>
__device__ inline int vq_exact_scan(const VqTables<SUB>& T, const double (&y)[SUB]) {
  double e1 = INFINITY;
  int k = 0;
  for (int c = 0; c < kCodes; ++c) {
    const double d = exact_dist<SUB>(T, y, c);
    if (d < e1) {
      e1 = d;
      k = c;
    }
  }
  return k;
}

template <int SUB>
__device__ inline int vq_search(const VqTables<SUB>& T, const double (&y)[SUB]) {
  float yf[SUB];
  float yn2 = 0.f;
#pragma unroll
  for (int i = 0; i < SUB; ++i) {
    yf[i] = (float)y[i];
    yn2 = fmaf(yf[i], yf[i], yn2);
  }
  float b1 = INFINITY, b2 = INFINITY;
  int i1 = 0;
#pragma unroll 8
  for (int c = 0; c < kCodes; ++c) {
    float d = T.cn[c];
#pragma unroll
    for (int i = 0; i < SUB; ++i) d = fmaf(T.neg2c[c][i], yf[i], d);
    const bool lt1 = d < b1;
    b2 = lt1 ? b1 : fminf(b2, d);
    i1 = lt1 ? c : i1;
    b1 = lt1 ? d : b1;
  }
  // Rounding-error window of the fp32 pass (inputs rounded to fp32, SUB fused steps, ||c||^2).
  const float M = T.cmax * T.cmax + 2.f * T.cmax * sqrtf(yn2);
  const float window = (8.f * (SUB + 3)) * 5.9604645e-8f * M;
  if (!(b2 - b1 > window)) i1 = vq_exact_scan<SUB>(T, y);
  return i1;
}

}  // namespace nsn
