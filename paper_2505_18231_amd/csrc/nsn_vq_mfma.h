// Nearest-codeword search (Eq. 1) with the distance contraction on the matrix cores.
//
// One v_mfma_f32_32x32x16_f16 produces, for 32 codewords (rows) and 32 sub-vectors (columns),
//   D = ||c||^2 - 2 c . (y_hi + y_lo) + ||y||^2 + margin      (fp32 accumulate)
// from fp16 operands: the codeword side holds [-2c | -2c | cn_hi cn_lo 1 1 0..] (SUB = 4) or
// [-2c | cn_hi cn_lo 1 1 0..] (SUB = 8, second pass for y_lo), the token side holds
// [y_hi | y_lo | 1 1 yn_hi yn_lo 0..].  Codewords are fp16 values, so -2c is exact; y, ||c||^2 and
// ||y||^2 are split into fp16 hi + lo parts (about 22 bits).  D > 0, so its bit pattern orders
// like an integer: the low 4 bits are replaced by the row slot and the best two keys are kept
// with a min3, a med3 and a min per pair of values.  If the runner-up is within the error window of the best
// (key granularity + fp32 rounding of the contraction), the decision is retaken in fp64 among the
// codewords inside that window, so the result equals the fp64 exhaustive search of the
// vector-ALU form.
#pragma once

#include "nsn_vq.h"

namespace nsn {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr float kVqMargin = 0.015625f;  // keeps every distance strictly positive

template <int SUB>
struct MfmaCodebook {
  h8 A[8];  // codeword-side operands of the eight 32-codeword blocks
};

// Build the codeword-side operands (call after vq_tables_fill; every lane of the wave).
template <int SUB>
__device__ inline void mfma_codebook_load(MfmaCodebook<SUB>& M, const VqTables<SUB>& T, int lane) {
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const int c = 32 * m + (lane & 31);
    h8 a;
    if (lane < 32) {
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = (_Float16)T.neg2c[c][e % SUB];
    } else {
      const float cn = T.cn[c];
      const _Float16 hi = (_Float16)cn;
      a[0] = hi;
      a[1] = (_Float16)(cn - (float)hi);
      a[2] = (_Float16)1.0f;
      a[3] = (_Float16)1.0f;
      a[4] = a[5] = a[6] = a[7] = (_Float16)0.0f;
    }
    M.A[m] = a;
  }
}

__device__ inline uint32_t pack_h2(_Float16 lo, _Float16 hi) {
  union {
    _Float16 h[2];
    uint32_t u;
  } cv;
  cv.h[0] = lo;
  cv.h[1] = hi;
  return cv.u;
}
__device__ inline h8 as_h8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  union {
    uint32_t u[4];
    h8 h;
  } cv;
  cv.u[0] = a, cv.u[1] = b, cv.u[2] = c, cv.u[3] = d;
  return cv.h;
}

// All 64 lanes call this; lane (token slot, sub-vector) layout as in the encoder: lanes [0,32) hold
// the sub-vectors of the first token set, lanes [32,64) those of the second.
template <int SUB>
__device__ inline int vq_search_mfma(const VqTables<SUB>& T, const MfmaCodebook<SUB>& M, const double (&y)[SUB],
                                     int lane) {
  constexpr int NP = SUB / 2;  // packed dwords per hi / lo part
  // token-side operand words of this lane's sub-vector (own: P, Q) and of lane ^ 32 (X, Qx)
  struct Words {
    uint32_t Phi[NP], Plo[NP], Xhi[NP], Xlo[NP], Q, Qx;
    float yn;
  };
  auto make_words = [&](const double (&yy)[SUB]) {
    Words w;
    _Float16 yh[SUB], yl[SUB];
    w.yn = 0.f;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      const float yf = (float)yy[i];
      yh[i] = (_Float16)yf;
      yl[i] = (_Float16)(yf - (float)yh[i]);
      w.yn = fmaf(yf, yf, w.yn);
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      w.Phi[i] = pack_h2(yh[2 * i], yh[2 * i + 1]);
      w.Plo[i] = pack_h2(yl[2 * i], yl[2 * i + 1]);
    }
    const float ynm = w.yn + kVqMargin;  // yn itself is needed for the window below
    const _Float16 ynh = (_Float16)ynm;
    w.Q = pack_h2(ynh, (_Float16)(ynm - (float)ynh));
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      w.Xhi[i] = __shfl_xor(w.Phi[i], 32, 64);
      w.Xlo[i] = __shfl_xor(w.Plo[i], 32, 64);
    }
    w.Qx = __shfl_xor(w.Q, 32, 64);
    return w;
  };
  const Words W = make_words(y);
  const float yn = W.yn;
  const uint32_t(&Phi)[NP] = W.Phi;
  const uint32_t(&Plo)[NP] = W.Plo;
  const uint32_t(&Xhi)[NP] = W.Xhi;
  const uint32_t(&Xlo)[NP] = W.Xlo;
  const uint32_t Q = W.Q, Qx = W.Qx;
  const bool lo_half = lane < 32;
  const uint32_t ONES = 0x3C003C00u;  // (1.0, 1.0)

  uint32_t k1 = 0u, k2 = 0u;  // best two keys of the sub-vector this lane owns
  int code = 0;
#pragma unroll
  for (int set = 0; set < 2; ++set) {
    const uint32_t* ph = (set == 0) ? Phi : Xhi;
    const uint32_t* pl = (set == 0) ? Plo : Xlo;
    const uint32_t qq = (set == 0) ? Qx : Q;
    h8 b1, b2;
    if constexpr (SUB == 4) {
      b1 = lo_half ? as_h8(ph[0], ph[1], pl[0], pl[1]) : as_h8(ONES, qq, 0u, 0u);
      b2 = b1;
    } else {
      b1 = lo_half ? as_h8(ph[0], ph[1], ph[2], ph[3]) : as_h8(ONES, qq, 0u, 0u);
      b2 = lo_half ? as_h8(pl[0], pl[1], pl[2], pl[3]) : as_h8(0u, 0u, 0u, 0u);
    }
    // keys are positive floats: unsigned-integer order equals float order (integer min avoids
    // the NaN canonicalisation a float min would add).  Two independent best-two chains
    // (even / odd blocks) keep a lone wave from serialising on one dependency chain.
    uint32_t ma1 = 0x7f000000u, ma2 = 0x7f000000u, mb1 = 0x7f000000u, mb2 = 0x7f000000u;
    int blka = 0, blkb = 1;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      f16v d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
      d = __builtin_amdgcn_mfma_f32_32x32x16_f16(M.A[m], b1, d, 0, 0, 0);
      if constexpr (SUB == 8) d = __builtin_amdgcn_mfma_f32_32x32x16_f16(M.A[m], b2, d, 0, 0, 0);
      uint32_t& m1r = (m & 1) ? mb1 : ma1;
      uint32_t& m2r = (m & 1) ? mb2 : ma2;
      int& blkr = (m & 1) ? blkb : blka;
      const uint32_t prev = m1r;
      // two keys at a time: the smallest of {best, a, b} is the new best, and the runner-up of everything
      // seen so far is the smaller of the old runner-up and the median of {best, a, b} (five instructions
      // per pair: two index insertions, min3, med3, min)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const uint32_t ua = (__float_as_uint(d[r]) & 0xFFFFFFF0u) | (uint32_t)r;
        const uint32_t ub = (__float_as_uint(d[r + 1]) & 0xFFFFFFF0u) | (uint32_t)(r + 1);
        const uint32_t mid = __float_as_uint(
            __builtin_amdgcn_fmed3f(__uint_as_float(m1r), __uint_as_float(ua), __uint_as_float(ub)));
        m2r = min(m2r, mid);
        m1r = min(m1r, min(ua, ub));
      }
      blkr = (m1r < prev) ? m : blkr;
    }
    const uint32_t m1 = min(ma1, mb1);
    const uint32_t m2 = min(max(ma1, mb1), min(ma2, mb2));
    const int blk = (mb1 < ma1) ? blkb : blka;
    const int r = (int)(m1 & 15u);
    const int mine = 32 * blk + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    // the other half of the wave scanned the other 128 codewords of the same sub-vectors
    const uint32_t o1 = __shfl_xor(m1, 32, 64), o2 = __shfl_xor(m2, 32, 64);
    const int ocode = __shfl_xor(mine, 32, 64);
    const uint32_t f1 = min(m1, o1);
    const uint32_t f2 = min(max(m1, o1), min(m2, o2));
    const int fcode = (o1 < m1) ? ocode : (o1 == m1 ? min(mine, ocode) : mine);
    if ((set == 0) == lo_half) {
      k1 = f1;
      k2 = f2;
      code = fcode;
    }
  }
  // error window: key granularity (16 ulp, truncated) + fp32 rounding of a 16-term contraction
  const float d1 = __uint_as_float(k1 & 0xFFFFFFF0u);
  const float d2 = __uint_as_float(k2 & 0xFFFFFFF0u);
  const float reach = T.cmax + sqrtf(yn);
  const float window = 2.f * (1.9073486e-6f * d2 + 24.f * 5.9604645e-8f * (reach * reach + kVqMargin));
  const bool need = !(d2 - d1 > window);
  if (__any(need)) {
    // Rare path, taken by the whole wave when any of its sub-vectors is undecided: repeat the
    // contraction and list, per undecided sub-vector, the codewords whose distance lies within
    // the window of the best one.  Every codeword that can be the true nearest is in that list
    // (its computed distance cannot exceed the best computed distance by more than the window).
    // Two entries (the usual case) are settled by two fp64 distances; more fall back to the
    // full fp64 scan.
    const uint32_t thr = need ? (__float_as_uint(d1 + window) | 15u) : 0u;  // bit pattern bound; 0 lists nothing
    const uint32_t thr_set[2] = {(uint32_t)__shfl((int)thr, lane & 31, 64),
                                 (uint32_t)__shfl((int)thr, (lane & 31) + 32, 64)};
    uint32_t listed[2];
    // The operand words are rebuilt from an opaque copy of y, so that nothing but y has to stay
    // in registers across the main pass for the sake of this rare path.
    double yy[SUB];
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      yy[i] = y[i];
      asm volatile("" : "+v"(yy[i]));
    }
    const Words R = make_words(yy);
#pragma unroll
    for (int set = 0; set < 2; ++set) {
      const uint32_t* ph = (set == 0) ? R.Phi : R.Xhi;
      const uint32_t* pl = (set == 0) ? R.Plo : R.Xlo;
      const uint32_t qq = (set == 0) ? R.Qx : R.Q;
      h8 b1, b2;
      if constexpr (SUB == 4) {
        b1 = lo_half ? as_h8(ph[0], ph[1], pl[0], pl[1]) : as_h8(ONES, qq, 0u, 0u);
        b2 = b1;
      } else {
        b1 = lo_half ? as_h8(ph[0], ph[1], ph[2], ph[3]) : as_h8(ONES, qq, 0u, 0u);
        b2 = lo_half ? as_h8(pl[0], pl[1], pl[2], pl[3]) : as_h8(0u, 0u, 0u, 0u);
      }
      // Branch- and compare-free listing with small immediates only (nothing for the compiler to
      // park in registers across the main pass): (thr - u) >> 31 is all ones exactly when u > thr
      // (both are bit patterns of positive floats, below 2^31); count and row offsets of the
      // REJECTED entries are summed per block, the listed ones follow by subtraction.
      uint32_t acc = 0u;  // count in bits 16.., sum of (index without the lane part) in bits 0..15
      float zero = 0.f;
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        // one block at a time: the next contraction starts from a zero that is ordered after this
        // block's sums, so the sixteen distances of a single block are all that is live here
        asm volatile("" : "+v"(zero), "+v"(acc));
        f16v d;
#pragma unroll
        for (int r = 0; r < 16; ++r) d[r] = zero;
        d = __builtin_amdgcn_mfma_f32_32x32x16_f16(M.A[m], b1, d, 0, 0, 0);
        if constexpr (SUB == 8) d = __builtin_amdgcn_mfma_f32_32x32x16_f16(M.A[m], b2, d, 0, 0, 0);
        int rej_cnt = 0, rej_off = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int out_mask = (int)(thr_set[set] - __float_as_uint(d[r])) >> 31;
          rej_cnt -= out_mask;
          rej_off += out_mask & (8 * (r >> 2) + (r & 3));
        }
        const uint32_t cnt = (uint32_t)(16 - rej_cnt);
        const uint32_t off = (uint32_t)(216 - rej_off);  // all sixteen rows: 4 * 8 * (0+1+2+3) + 4 * (0+1+2+3)
        acc += (cnt << 16) + off + cnt * (32u * m);
      }
      acc += (acc >> 16) * (4u * (lane >> 5));  // this lane's rows sit 4 * (lane / 32) further down
      listed[set] = acc + (uint32_t)__shfl_xor((int)acc, 32, 64);
    }
    if (need) {
      const uint32_t mine = lo_half ? listed[0] : listed[1];
      const int other = (int)(mine & 0xFFFFu) - code;
      if ((mine >> 16) == 2u && other >= 0 && other < kCodes) {
        const double e_code = exact_dist<SUB>(T, y, code), e_other = exact_dist<SUB>(T, y, other);
        if (e_other < e_code || (e_other == e_code && other < code)) code = other;
      } else {
        code = vq_exact_scan<SUB>(T, y);
      }
    }
  }
  return code;
}

}  // namespace nsn
