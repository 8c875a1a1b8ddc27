// Device-side helpers shared by the encode / decode / codebook kernels (gfx950, wave64).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nsn.h"

namespace nsn {

constexpr int kHeadDim = 128;
constexpr int kCodes = 256;
constexpr double kInvSqrtD = 0.08838834764831844055;  // 1/sqrt(128)
constexpr double kSqrtD = 11.31370849898476039041;     // sqrt(128)

// ---- cache addressing -----------------------------------------------------------------
struct CacheView {
  uint8_t* codes;
  __half2* norms;
  __half* means;
  const int32_t* block_table;
};

// fp16 rows of the most recent tokens that are not coded yet (Sec. 3.2 "Residual"):
// [sequence][kv head][capacity][head_dim]; k == nullptr means there is none
struct ResidualView {
  const __half* k;
  const __half* v;
  const int32_t* lens;  // valid rows per sequence
  int capacity;         // <= 64
};

constexpr int kSignCodes = 65536;  // n_codes value that selects the sign + index format
constexpr int kCounterStrideInts = 64;  // decode arrival counters: one per 256-byte line

// Table of nsn_build_rope_table (byte offsets): fp16 hi / lo of (cos, sin)(j * inv_freq[i]) as
// rows [j][128] (64 cosines, then 64 sines), the same angles in fp64 as (cos, sin) pairs [j][i],
// then one 1536-byte record per 64-token block: (cos, sin)(64 * block * inv_freq[i]) as 64 fp32
// pairs followed by 64 fp64 pairs.
constexpr int kRopeHiOff = 0, kRopeLoOff = 16384, kRopeInOff = 32768, kRopeBlkOff = 32768 + 65536;
constexpr int kRopeBlkStride = 1536, kRopeBlk64 = 512;

// Double quantization (side_bits = 4): byte sizes of a 64-token norms record and of a mean record
constexpr int kDqNormRec = 164, kDqNormCodes = 128, kDqNormPar = 160;
constexpr int kDqMeanRec = 80, kDqMeanPar = 64;

struct Geometry {
  int tiled;                  // 1: codes in the tiled layout (64-token blocks, see k_code_offset_tiled)
  int dq;                     // 1: norms and means are stored in 4 bits (records above)
  const unsigned char* rope;  // table of nsn_build_rope_table, or nullptr (keys coded as given)
  int sign;         // 1: an 8-dim sub-vector is an index byte plus a sign byte (byte rows 0..15 / 16..31)
  int J;            // code bytes per token
  int n_q_heads, n_kv_heads;
  int group_size;   // 0 = one group
  int n_groups_max; // mean vectors per (sequence, kv-head)
  int page_tokens;  // tokens per placement unit: page_size if paged, else max_len
  int pages_per_seq;  // max_len / page_size if paged, else 1
  int paged;
  // log2 of group_size / page_tokens when they are powers of two (the usual case), else -1: the
  // kernels index groups and pages once or more per 64 tokens, and a division by a run-time value
  // costs about 35 scalar instructions
  int group_shift, page_shift;
};

// Byte offset, inside one placement unit, of the code of (token t of the unit, sub-vector j).
// K: token-major (a lane that owns a token reads its J bytes in one go).
// V: blocks of J tokens, sub-vector-major inside a block (a lane that owns a sub-vector reads
//    the codes of J consecutive tokens in one go).
__host__ __device__ inline int64_t k_code_offset(int J, int64_t t, int j) { return t * J + j; }
__host__ __device__ inline int64_t v_code_offset(int J, int64_t t, int j) {
  return (t / J) * (int64_t)(J * J) + (int64_t)j * J + (t % J);
}

// Tiled layout (the formats read by dec_tile_kernel): 64-token blocks of 64 * NSV bytes (NSV = sub-vectors
// per token), one run of NSV bytes per lane of the wave that reads the block (lane = 16 hi + lo):
//   K: lane = 16 * (j / QS) + t % 16, byte (t % 64 / 16) * QS + j % QS           (QS = NSV / 4)
//      - a lane holds one 32-channel quarter of tokens t % 16 of the block's four 16-token tiles
//   V: lane = 16 * (t % 16 / 4) + 4 * (t % 4) + j % 4, byte (t % 64 / 16) * QS + j / 4
//      - a lane holds sub-vectors j % 4 == const of four tokens that are 16 apart
__host__ __device__ inline int64_t k_code_offset_tiled(int NSV, int64_t t, int j) {
  const int QS = NSV / 4, tb = (int)(t & 63);
  const int lane = 16 * (j / QS) + (tb & 15);
  return (t >> 6) * (int64_t)(64 * NSV) + lane * NSV + (tb >> 4) * QS + j % QS;
}
__host__ __device__ inline int64_t v_code_offset_tiled(int NSV, int64_t t, int j) {
  const int QS = NSV / 4, tb = (int)(t & 63);
  const int lane = 16 * ((tb & 15) >> 2) + 4 * (tb & 3) + (j & 3);
  return (t >> 6) * (int64_t)(64 * NSV) + lane * NSV + (tb >> 4) * QS + (j >> 2);
}
// the layout a cache of geometry g uses
__host__ __device__ inline int64_t code_offset(bool tiled, bool value, int J, int64_t t, int j) {
  if (tiled) return value ? v_code_offset_tiled(J, t, j) : k_code_offset_tiled(J, t, j);
  return value ? v_code_offset(J, t, j) : k_code_offset(J, t, j);
}

// Index (in tokens) of the first token of the placement unit holding token t of sequence b.
__device__ inline int page_of(const Geometry& g, int t) {
  return g.page_shift >= 0 ? t >> g.page_shift : t / g.page_tokens;
}
__device__ inline int64_t unit_token_base(const Geometry& g, const int32_t* block_table, int b, int h,
                                          int t) {
  int64_t page = b;
  if (g.paged) page = block_table[(int64_t)b * g.pages_per_seq + page_of(g, t)];
  return (page * g.n_kv_heads + h) * (int64_t)g.page_tokens;
}
__device__ inline int token_in_unit(const Geometry& g, int t) {
  if (!g.paged) return t;
  return g.page_shift >= 0 ? t & (g.page_tokens - 1) : t % g.page_tokens;
}
__device__ inline int group_of(const Geometry& g, int t) {
  if (g.group_size <= 0) return 0;
  return g.group_shift >= 0 ? t >> g.group_shift : t / g.group_size;
}

// Double quantization: record of the 64-token block holding token t of a placement unit that starts at
// token index `base`; mean record of (unit-relative) group gidx
__device__ inline unsigned char* dq_norm_rec(const CacheView& cv, int64_t base, int tin) {
  return reinterpret_cast<unsigned char*>(cv.norms) + ((base + tin) >> 6) * kDqNormRec;
}
__device__ inline unsigned char* dq_mean_rec(const CacheView& cv, int64_t mean_index) {
  return reinterpret_cast<unsigned char*>(cv.means) + mean_index * kDqMeanRec;
}

// ---- numeric helpers ------------------------------------------------------------------
// fp64 -> fp16, round to nearest even in a single rounding: go through fp32 with
// round-to-odd (sticky bit in the last place), then the hardware fp32 -> fp16 rounding.
__device__ inline __half f64_to_f16(double x) {
  float f = (float)x;
  const double r = x - (double)f;
  if (r != 0.0 && f != 0.0f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 1u) == 0u) {
      const bool grow = (r > 0.0) == (f > 0.0f);
      u = grow ? u + 1u : u - 1u;
      f = __uint_as_float(u);
    }
  }
  return __float2half_rn(f);
}

// Value of lane (lane ^ M): DPP moves inside a 16-lane row (no LDS traffic), a bpermute across rows.
template <int CTRL, int BANK>
__device__ __forceinline__ int dpp_i32(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, 0xf, BANK, false);
}
// (every lane has a valid source in these patterns and the callers run with all lanes active, so the
// destination needs no defined previous value: the form without one saves the move that would set it)
template <int CTRL, int BANK>
__device__ __forceinline__ int dpp_mov_i32(int v) {
  return __builtin_amdgcn_mov_dpp(v, CTRL, 0xf, BANK, true);
}
template <int M>
__device__ __forceinline__ int xor_lane_i32(int v) {
  if constexpr (M == 1) {
    return dpp_mov_i32<0xB1, 0xf>(v);  // quad_perm [1,0,3,2]
  } else if constexpr (M == 2) {
    return dpp_mov_i32<0x4E, 0xf>(v);  // quad_perm [2,3,0,1]
  } else if constexpr (M == 4) {
    const int t = dpp_mov_i32<0x104, 0x5>(v);  // row_shl:4 into lanes whose bit 2 is clear
    return dpp_i32<0x114, 0xa>(t, v);          // row_shr:4 into lanes whose bit 2 is set
  } else if constexpr (M == 8) {
    return dpp_mov_i32<0x128, 0xf>(v);  // row_ror:8
  } else {
    return __shfl_xor(v, M, 64);
  }
}
template <int M>
__device__ __forceinline__ float xor_lane(float v) {
  return __builtin_bit_cast(float, xor_lane_i32<M>(__builtin_bit_cast(int, v)));
}
template <int M>
__device__ __forceinline__ double xor_lane(double v) {
  const long long u = __builtin_bit_cast(long long, v);
  const unsigned lo = (unsigned)xor_lane_i32<M>((int)(u & 0xffffffffll));
  const unsigned hi = (unsigned)xor_lane_i32<M>((int)(u >> 32));
  return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)lo);
}
// Butterfly sum over groups of W lanes (W a power of two <= 64); every lane gets the total.
template <int W, typename T>
__device__ __forceinline__ T xor_sum_w(T v) {
  if constexpr (W > 1) v += xor_lane<1>(v);
  if constexpr (W > 2) v += xor_lane<2>(v);
  if constexpr (W > 4) v += xor_lane<4>(v);
  if constexpr (W > 8) v += xor_lane<8>(v);
  if constexpr (W > 16) v += xor_lane<16>(v);
  if constexpr (W > 32) v += xor_lane<32>(v);
  return v;
}

template <typename T>
__device__ inline T xor_sum(T v, int width) {  // butterfly sum over groups of `width` lanes
  for (int m = 1; m < width; m <<= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ inline float wave_max(float v) {
  for (int m = 1; m < 64; m <<= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

}  // namespace nsn
