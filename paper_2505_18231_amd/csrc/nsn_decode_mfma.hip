// Decode attention over the coded cache (App. B): matrix-core form for gfx950.
//
// Same arithmetic as the lookup-table kernel, arranged for the CDNA4 execution units:
//   * every lane owns one token of a 64-token group; its K code bytes index a codebook table in
//     LDS that is replicated once per bank group, so the 64 gathers of a wave never conflict;
//   * the gathered fp16 codeword IS the B operand of v_mfma_f32_4x4x4_16B_f16 (k = the four
//     channels of one sub-vector, column = the lane's token); the rotated query, split into
//     fp16 hi + lo parts, is the A operand, broadcast from one 4-lane block to all sixteen
//     (cbsz / abid), so HT(q) . C[code] accumulates in fp32 with ~22 significant bits and the
//     lane ends up holding its token's score for up to four query heads - no table per query;
//   * softmax weights are formed per lane (lazy running max per head: acc is rescaled only
//     when a score exceeds the running max by more than 2^5);
//   * for the value side a lane owns one sub-vector of 32 (or 16) tokens; four gathered
//     codewords are transposed in registers (v_perm_b32) into "four tokens of one channel"
//     B operands, the fp16 weights of those four tokens are the broadcast A operand, and the
//     fp32 accumulator is out_rot[head][channel] in the rotated domain;
//   * one workgroup per (split, kv head, sequence); the last workgroup of a (kv head, sequence)
//     to finish merges the splits (running max / sum), applies the single inverse Hadamard per
//     head, adds the mean-vector term and writes the output - no second launch.
#include <cstdlib>
#include <type_traits>

#include "nsn_host.h"

namespace nsn {

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8d __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kPartialStrideM = 2 * kHeadDim + 2;  // rotated acc, mean-term acc, m (log2 units), l
constexpr float kLazyMaxLog2 = 5.0f;               // rescale only when a score beats the running max by 2^5
// The fp16 softmax weights are p a^v 2^10 / A with A a running power of two >= every a^v seen so far: they
// lie in [0, 2^15] whatever the scale of the values is (the first Normalize of Sec. 3.2 keeps every token
// norm apart, so attention must not depend on it either); the accumulators are in units of A / 2^10.
constexpr float kWeightScaleM = 1024.0f;
constexpr int kTableBytes = 65536;

template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }  // 2^-inf = 0
__device__ __forceinline__ uint32_t perm_b32(uint32_t s0, uint32_t s1, uint32_t sel) {
  return __builtin_amdgcn_perm(s0, s1, sel);
}
__device__ __forceinline__ h4 as_h4(uint32_t lo, uint32_t hi) {
  union {
    uint32_t u[2];
    h4 h;
  } cv;
  cv.u[0] = lo;
  cv.u[1] = hi;
  return cv.h;
}
template <int CTRL>
__device__ __forceinline__ float dpp_quad(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ float dpp_row(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float read_lane(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
// Wave-wide reductions on the vector ALU (no LDS traffic); the result is uniform.
// quad xor 1, quad xor 2, mirror within 8 lanes, mirror within 16 lanes: every lane holds its
// row's result; then lane 15 of a row is broadcast into the next row (rows 1 and 3), lane 31 into
// rows 2 and 3, and lane 63 holds the result of the wave.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_row_masked(float keep, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, keep), __builtin_bit_cast(int, v),
                                                               CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_u(float v) {
  v += dpp_row<0xB1>(v);
  v += dpp_row<0x4E>(v);
  v += dpp_row<0x141>(v);
  v += dpp_row<0x140>(v);
  v += dpp_row_masked<0x142, 0xA>(0.f, v);  // rows 1, 3 += row 0, 2
  v += dpp_row_masked<0x143, 0xC>(0.f, v);  // rows 2, 3 += rows 0 + 1
  return read_lane(v, 63);
}
__device__ __forceinline__ float wave_max_u(float v) {
  v = fmaxf(v, dpp_row<0xB1>(v));
  v = fmaxf(v, dpp_row<0x4E>(v));
  v = fmaxf(v, dpp_row<0x141>(v));
  v = fmaxf(v, dpp_row<0x140>(v));
  v = fmaxf(v, dpp_row_masked<0x142, 0xA>(v, v));
  v = fmaxf(v, dpp_row_masked<0x143, 0xC>(v, v));
  return read_lane(v, 63);
}

// Device-scope stores / loads: coherent across the chip's L2 slices without cache maintenance.
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS reads by absolute LDS byte address (the codebook table starts at LDS address 0).
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ uint2 lds_read64(uint32_t addr) {
  typedef uint32_t u2 __attribute__((ext_vector_type(2)));
  const u2 v = *(const u2 __attribute__((address_space(3)))*)(addr);
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint4 lds_read128(uint32_t addr) {
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  const u4 v = *(const u4 __attribute__((address_space(3)))*)(addr);
  return make_uint4(v.x, v.y, v.z, v.w);
}
#else
__device__ __forceinline__ uint2 lds_read64(uint32_t) { return make_uint2(0, 0); }
__device__ __forceinline__ uint4 lds_read128(uint32_t) { return make_uint4(0, 0, 0, 0); }
#endif

// Transpose a 4x4 fp32 tile held as x[0..3] across the four lanes of every quad:
// afterwards lane i of a quad holds x[k] = (old x[i] of lane k).
__device__ __forceinline__ void quad_transpose(float (&x)[4], int lane) {
  const bool odd = lane & 1, up = lane & 2;
  {
    const float s01 = odd ? x[0] : x[1], s23 = odd ? x[2] : x[3];
    const float r01 = dpp_quad<0xB1>(s01), r23 = dpp_quad<0xB1>(s23);  // lane ^ 1
    if (odd) {
      x[0] = r01;
      x[2] = r23;
    } else {
      x[1] = r01;
      x[3] = r23;
    }
  }
  {
    const float s0 = up ? x[0] : x[2], s1 = up ? x[1] : x[3];
    const float r0 = dpp_quad<0x4E>(s0), r1 = dpp_quad<0x4E>(s1);  // lane ^ 2
    if (up) {
      x[0] = r0;
      x[1] = r1;
    } else {
      x[2] = r0;
      x[3] = r1;
    }
  }
}

// LDS plan (dynamic, starts at LDS address 0):
//   [0, 64 KiB)        codebook table: entry (code c, copy p) at c * 256 + p * (2 * SUB) bytes,
//                      32 copies of 8 B (SUB = 4) or 16 copies of 16 B (SUB = 8);
//                      after the main loop the same bytes hold the per-wave accumulators
//   then 8.25 KiB      staged codewords, unrotated query (read again when a wave enters another
//                      Shift group), rotated query, q . o^k of the split's first group
//   then (NW+1)*2 KiB  mean-vector term of every wave, accm[NW + 1][4][128] (slot NW belongs to
//                      the residual wave, present only in residual launches)
//   tail               per-wave (m, l), the "last workgroup" flag
//   ROPE only: 32 KiB  fp16 hi and lo parts of (cos, sin)(j * inv_freq[i]), rows of 256 bytes whose
//                      16-byte chunks are XOR-swizzled by the row number (conflict-free operand reads)
//              32 KiB  per wave, q . RoPE_t(o^k) of the 64 tokens of its next four groups, four heads each
// One workgroup of 8 (or 11) main waves per compute unit shares a single table (about 92 of the 160 KiB).
template <int SUB, int NW, bool SGN = false, bool ROPE = false>
struct DecSmem {
  // sign + index format: a 4 KiB table of sign masks sits in front of the codebook table
  static constexpr int kSignLutBytes = SGN ? 4096 : 0;
  static constexpr int kTable = kTableBytes + kSignLutBytes;
  static constexpr int kQoTabGroups = 64;  // q . o^k of up to 64 Shift groups of a split, four heads each
  static constexpr int kStageBytes = ((kCodes * 2 * SUB + 2 * 4 * kHeadDim * 4 + 16 + kQoTabGroups * 16) + 255) & ~255;
  static constexpr int kRaccBytes = NW * (64 / (kHeadDim / SUB)) * 4 * kHeadDim * 4;
  // (the per-wave accumulators reuse the table and, where they are larger - 11 waves of 8-dim
  // sub-vectors -, the staging area behind it: both are dead once the main loop is over)
  static constexpr int kAccmOffset =
      kTable + kStageBytes > ((kRaccBytes + 255) & ~255) ? kTable + kStageBytes : ((kRaccBytes + 255) & ~255);
  static constexpr int kAccmBytes = (NW + 1) * 4 * kHeadDim * 4;  // + the residual wave's slot
  static constexpr int kTailBytes = (2 * (NW + 1) * 4 + 4 + 4 * kHeadDim) * 4;
  static constexpr bool kTailInTable = kRaccBytes + kTailBytes <= kTable;
  static constexpr int kTailOffset = kTailInTable ? kRaccBytes : kAccmOffset + kAccmBytes;
  static constexpr int kPlainBytes = kAccmOffset + kAccmBytes + (kTailInTable ? 0 : kTailBytes);
  static constexpr int kRopeBatch = 4;  // groups per wave whose mean term is formed in one go
  static constexpr int kRopeTabOffset = (kPlainBytes + 255) & ~255;
  static constexpr int kRopeTabBytes = 2 * 64 * 256;
  static constexpr int kRopeDotOffset = kRopeTabOffset + kRopeTabBytes;
  static constexpr int kRopeDotBytes = NW * kRopeBatch * 64 * 16;
  static constexpr int kBytes = ROPE ? kRopeDotOffset + kRopeDotBytes : kPlainBytes;
  static_assert(kBytes <= 160 * 1024, "LDS of one compute unit");
  // Residual launches of the instances that have the room stage the fp16 residual rows in LDS: key rows
  // with a padded stride (a lane reads its own token's row), value rows as they are.
  static constexpr bool kResInLds = !ROPE;
  static constexpr int kResKStride = SUB == 4 ? 264 : 272;
  static constexpr int kResOffset = (kBytes + 255) & ~255;
  static constexpr int kResBytes = kResInLds ? 64 * kResKStride + 64 * 256 : 0;
  static_assert(kResOffset + kResBytes <= 160 * 1024, "LDS of one compute unit");
  static_assert(kRaccBytes <= kAccmOffset, "per-wave accumulators must end below the mean-term accumulators");
};

// R = query heads per kv head handled by the kernel instance (1, 2 or 4; three heads run as 4).
// With R <= 2 the fp16 hi and lo parts of the rotated query share the four MFMA rows
// (rows [0,R) = hi, rows [R,2R) = lo), so one MFMA per slot suffices.
// SGN = the sign + index format (Sec. 3.4): SUB = 8, code bytes [0,16) of a token are indices into a
// codebook of magnitudes, bytes [16,32) the sign bytes; a gathered codeword gets its sign bits from
// two 8-byte mask entries (one per sign nibble) of a small replicated table, XORed in before the MFMA.
// ROPE = the keys were normalised before the rotary embedding (Sec. 3.2 "NSN applied to key and value"):
// the mean term of the score is b_t * q . RoPE_t(o) (App. B).  With t = 64 * block + j and the pair
// (i, i + 64) of channels,   q . RoPE_t(o) = sum_i cos(j w_i) A'_i + sin(j w_i) B'_i,   where
//   A_i = q_i o_i + q_i' o_i',  B_i = q_i' o_i - q_i o_i'   (i' = i + 64)
//   A'_i = A_i c_i + B_i s_i,   B'_i = B_i c_i - A_i s_i,   (c_i, s_i) = (cos, sin)(64 * block * w_i):
// a [64 tokens x 128] x [128 x heads] contraction whose token-side operand is the same for every
// group.  A wave forms it for its next four groups at once with v_mfma_f32_16x16x32_f16 (rows = (group,
// head), columns = 16 tokens; fp16 hi + lo parts on both sides, three products), leaves the 64 x 4
// results per group in LDS, and the main loop reads one 16-byte entry per lane and group.
// DQ = double quantization (Sec. 3.5): norms and means are 4-bit codes with fp16 (min, step) per group;
// they are expanded where the fp16 forms are unpacked, everything downstream is unchanged.
template <int SUB, int NW, int R, bool SGN = false, bool ROPE = false, bool DQ = false>
__global__ __launch_bounds__((NW + 1) * 64) void dec_mfma_kernel(Geometry g, const __half* __restrict__ codebook,
                                                           const __half* __restrict__ q, CacheView kc,
                                                           CacheView vc, const int32_t* __restrict__ seq_lens,
                                                           float scale_log2e, int n_splits, int per,
                                                           float* partial, int* counters,
                                                           ResidualView res, int head_off, int r_pass,
                                                           float* __restrict__ out) {
  static_assert(!SGN || SUB == 8, "the sign + index format is defined on 8-dim sub-vectors");
  constexpr int NSV = kHeadDim / SUB;         // sub-vectors per token
  constexpr int J = SGN ? 2 * NSV : NSV;      // code bytes per token
  constexpr int IW = NSV / 4;                 // index dwords per lane (K: one token; V: one sub-vector of NSV tokens)
  constexpr int KW = SGN ? 2 * IW : IW;       // code dwords per lane (indices, then sign bytes)
  constexpr int LV = NSV;                     // lanes per value-side token part (one lane per sub-vector)
  constexpr int NPART = 64 / LV;              // value-side token parts of a 64-token group
  constexpr uint32_t TB = SGN ? 4096u : 0u;   // LDS address of the codebook table
  constexpr int CBSZ_V = (SUB == 4) ? 3 : 2;
  constexpr int NT = NW * 64;
  constexpr bool PACK = (R <= 2);  // hi and lo rows in one A operand
  constexpr int CH = SGN ? 2 : 8;  // key-side gathers in flight per chunk (a sign-format gather is 8 registers)
  using SM = DecSmem<SUB, NW, SGN, ROPE>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  unsigned char* const sm_table = smem_raw;
  unsigned char* const sm_stage = smem_raw + SM::kTable;
  float(*const sm_q_orig)[kHeadDim] = reinterpret_cast<float(*)[kHeadDim]>(sm_stage + kCodes * 2 * SUB);
  float(*const sm_q_had)[kHeadDim] = sm_q_orig + 4;
  float(*const sm_q_keep)[kHeadDim] = sm_q_orig;  // stays valid for the whole kernel
  float* const sm_qo_first = &sm_q_had[4][0];  // q . o^k of the split's first Shift group, four heads
  float4* const sm_qo_tab = reinterpret_cast<float4*>(sm_qo_first + 4);  // [kQoTabGroups], 16-byte aligned
  float(*const sm_accm)[4][kHeadDim] = reinterpret_cast<float(*)[4][kHeadDim]>(smem_raw + SM::kAccmOffset);
  float(*const sm_wave_m)[4] = reinterpret_cast<float(*)[4]>(smem_raw + SM::kTailOffset);  // after the loop
  float(*const sm_wave_l)[4] = sm_wave_m + (NW + 1);
  int* const sm_is_last = reinterpret_cast<int*>(sm_wave_l + (NW + 1));
  unsigned char* const sm_rope_tab = smem_raw + SM::kRopeTabOffset;  // ROPE only
  float4(*const sm_rope_dot)[SM::kRopeBatch][64] =
      reinterpret_cast<float4(*)[SM::kRopeBatch][64]>(smem_raw + SM::kRopeDotOffset);

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  // this launch handles query heads [head_off, head_off + r_pass) of every kv head (r_pass <= 4;
  // more than four heads per kv head run as two launches)
  const int r = r_pass;
  const int hq0 = h * (g.n_q_heads / g.n_kv_heads) + head_off;  // first query head of this workgroup
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // per-wave bookkeeping on the scalar unit
  // Launches with a residual carry one more wave (index NW): it handles the fp16 residual tokens
  // while the NW main waves run their loops, takes no part in the cooperative prologue work and
  // joins the others at every barrier.
  const int n_waves = (int)(blockDim.x >> 6);  // NW or NW + 1
  const bool main_wave = wave < NW;
  const int t0 = split * per;
  const int64_t mean_base = (int64_t)(b * g.n_kv_heads + h) * g.n_groups_max;

  // One 64-token group's cache bytes as this lane needs them: the J code bytes of its K token,
  // the J code bytes (J consecutive tokens) of its V sub-vector, the two norm pairs, and this
  // lane's two channels of the group's Shift vectors.
  struct Side {  // side information of the lane's token and the lane's two channels of the group's Shift vectors
    __half2 nk, nv, ok2, ov2;  // fp16 form: (a, b) of the K / V token, channels 2 lane, 2 lane + 1 of o^k / o^v
    // 4-bit form (DQ):
    uint32_t ka, va;    // a' = fp16(s2 alpha) of the token (low 16 bits)
    uint32_t kq, vq;    // byte holding the token's 4-bit s1 code (even token = low nibble)
    __half2 kp, vp;     // (min, step) of the 64-token block's s1 codes
    uint32_t okq, ovq;  // byte holding the lane's two 4-bit mean codes
    __half2 okp, ovp;   // (min, step) of the lane's 32-channel group
  };
  struct Grp {
    uint32_t kcode[KW], vcode[KW];
    Side s;
  };
  auto half_bits = [](uint32_t u) -> float { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu)); };
  auto lvl = [](__half2 par, uint32_t code) -> float {  // min + step * code
    return fmaf(__high2float(par), (float)code, __low2float(par));
  };
  // per-lane byte offsets (32-bit) that are added to wave-uniform 64-bit bases
  const uint32_t k_lane_off = lane * J;
  // value side: plain formats keep a sub-vector's NSV tokens contiguous (blocks of NSV tokens); the sign
  // format has blocks of 32 tokens with 32 byte rows: 16 tokens of index row j, their signs 16 rows on
  const uint32_t v_lane_off = SGN ? ((lane / LV) >> 1) * (J * J) + (lane % LV) * J + ((lane / LV) & 1) * 16
                                  : (lane / LV) * (J * J) + (lane % LV) * J;
  const uint32_t lane_x4 = lane * 4;
  // The three parts of a group's bytes can be loaded separately: the sign-format instances, which
  // are short of registers, refill the code registers in place as soon as their phase is over; the
  // others fetch the whole next group one iteration ahead into a second set (longer prefetch
  // distance: measured 0.7 us faster on the 38 MB shape).
  // A group that does not exist (`real` false: the wave's list has ended) is loaded all the same, from the first
  // bytes of every array (one cache line per instruction; nothing of it is used).  Loads that are only issued
  // under a condition make the number of loads behind a given one depend on the path; the compiler's wait
  // counts then take the smallest, and a wait for this group's bytes also waits for the next group's.
  auto group_base = [&](const int32_t* block_table, int tg, bool real) -> int64_t {  // wave-uniform
    return real ? unit_token_base(g, block_table, b, h, tg) + token_in_unit(g, tg) : 0;
  };
  auto load_k_codes = [&](int gi, bool real, Grp& G) {
    const int tg = t0 + (gi << 6);
    const int64_t kbase = group_base(kc.block_table, tg, real);
    const uint4* kp = reinterpret_cast<const uint4*>(kc.codes + kbase * J + (real ? k_lane_off : 0u));
#pragma unroll
    for (int w4 = 0; w4 < KW / 4; ++w4) {
      const uint4 kv4 = kp[w4];
      G.kcode[4 * w4] = kv4.x, G.kcode[4 * w4 + 1] = kv4.y, G.kcode[4 * w4 + 2] = kv4.z, G.kcode[4 * w4 + 3] = kv4.w;
    }
  };
  auto load_v_codes = [&](int gi, bool real, Grp& G) {
    const int tg = t0 + (gi << 6);
    const int64_t vbase = group_base(vc.block_table, tg, real);
    const uint4* vp = reinterpret_cast<const uint4*>(vc.codes + vbase * J + (real ? v_lane_off : 0u));
#pragma unroll
    for (int w4 = 0; w4 < KW / 4; ++w4) {
      // sign format: the value side's second 16 bytes are the sign row, NSV rows of J bytes further on
      const uint4 vv4 = (SGN && w4 == 1) ? vp[NSV * J / 16] : vp[w4];
      G.vcode[4 * w4] = vv4.x, G.vcode[4 * w4 + 1] = vv4.y, G.vcode[4 * w4 + 2] = vv4.z, G.vcode[4 * w4 + 3] = vv4.w;
    }
  };
  auto load_side = [&](int gi, bool real, Side& S) {
    const int tg = t0 + (gi << 6);
    const int64_t kbase = group_base(kc.block_table, tg, real), vbase = group_base(vc.block_table, tg, real);
    const int64_t mgrp = real ? mean_base + group_of(g, tg) : 0;  // wave-uniform
    const uint32_t ln = real ? (uint32_t)lane : 0u, lx4 = 4 * ln;  // (a missing group: every lane reads the same bytes)
    if constexpr (DQ) {
      const unsigned char* kr = reinterpret_cast<const unsigned char*>(kc.norms) + (kbase >> 6) * kDqNormRec;
      const unsigned char* vr = reinterpret_cast<const unsigned char*>(vc.norms) + (vbase >> 6) * kDqNormRec;
      S.ka = *reinterpret_cast<const uint16_t*>(kr + 2 * ln);
      S.va = *reinterpret_cast<const uint16_t*>(vr + 2 * ln);
      S.kq = kr[kDqNormCodes + (ln >> 1)];
      S.vq = vr[kDqNormCodes + (ln >> 1)];
      S.kp = *reinterpret_cast<const __half2*>(kr + kDqNormPar);
      S.vp = *reinterpret_cast<const __half2*>(vr + kDqNormPar);
      const int64_t mo = mgrp * kDqMeanRec;
      const unsigned char* km = reinterpret_cast<const unsigned char*>(kc.means) + mo;
      const unsigned char* vm = reinterpret_cast<const unsigned char*>(vc.means) + mo;
      S.okq = km[ln];
      S.ovq = vm[ln];
      S.okp = *reinterpret_cast<const __half2*>(km + kDqMeanPar + 4 * (ln >> 4));
      S.ovp = *reinterpret_cast<const __half2*>(vm + kDqMeanPar + 4 * (ln >> 4));
    } else {
      S.nk = *reinterpret_cast<const __half2*>(reinterpret_cast<const unsigned char*>(kc.norms + kbase) + lx4);
      S.nv = *reinterpret_cast<const __half2*>(reinterpret_cast<const unsigned char*>(vc.norms + vbase) + lx4);
      const int64_t mo = mgrp * kHeadDim;
      S.ok2 = *reinterpret_cast<const __half2*>(reinterpret_cast<const unsigned char*>(kc.means + mo) + lx4);
      S.ov2 = *reinterpret_cast<const __half2*>(reinterpret_cast<const unsigned char*>(vc.means + mo) + lx4);
    }
  };
  // the lane's two channels of a Shift vector as floats
  auto mean_pair = [&](const Side& S, bool key, float& o0, float& o1) {
    if constexpr (DQ) {
      const uint32_t q8 = key ? S.okq : S.ovq;
      const __half2 par = key ? S.okp : S.ovp;
      o0 = lvl(par, q8 & 15u);
      o1 = lvl(par, (q8 >> 4) & 15u);
    } else {
      const __half2 o2 = key ? S.ok2 : S.ov2;
      o0 = __low2float(o2);
      o1 = __high2float(o2);
    }
  };
  auto load_group = [&](int gi, bool real, Grp& G) {
    load_k_codes(gi, real, G);
    load_v_codes(gi, real, G);
    load_side(gi, real, G.s);
  };

  // ROPE: global operands of one batch of the mean term (four groups gi0, gi0 + NW, ...).  The four
  // lanes of a quad own the four heads of one group; for the loads they split the group's 16 pairs
  // (i, i + 64) of this lane's channel range: lane c of the quad takes four pairs of the mean row
  // (fp16) and of the block's (cos, sin) row (fp32).
  struct RopeIn {
    uint2 oa, ob;      // fp16 form: four channels from i0 and from 64 + i0
    uint32_t oaq, obq; // 4-bit form: their codes (two bytes each) ...
    __half2 oap, obp;  // ... and the (min, step) of their 32-channel groups
    float4 c01, c23;
  };
  auto rope_load = [&](int gi0, RopeIn& in) {
    const int m = lane & 15, bi = m >> 2, c = m & 3, kq = lane >> 4;
    // blocks past the sequence end are clamped into the tables (their results are never read)
    const int tg = min(t0 + ((gi0 + NW * bi) << 6), g.page_tokens * g.pages_per_seq - 64);
    const unsigned char* rec = g.rope + kRopeBlkOff + (int64_t)(tg >> 6) * kRopeBlkStride;
    const int i0 = 32 * (c >> 1) + 8 * kq + 4 * (c & 1);
    if constexpr (DQ) {
      const unsigned char* mr = reinterpret_cast<const unsigned char*>(kc.means) + (mean_base + group_of(g, tg)) * kDqMeanRec;
      in.oaq = *reinterpret_cast<const uint16_t*>(mr + (i0 >> 1));
      in.obq = *reinterpret_cast<const uint16_t*>(mr + ((64 + i0) >> 1));
      in.oap = *reinterpret_cast<const __half2*>(mr + kDqMeanPar + 4 * (i0 >> 5));
      in.obp = *reinterpret_cast<const __half2*>(mr + kDqMeanPar + 4 * ((64 + i0) >> 5));
    } else {
      const __half* orow = kc.means + (mean_base + group_of(g, tg)) * kHeadDim;
      in.oa = *reinterpret_cast<const uint2*>(orow + i0);
      in.ob = *reinterpret_cast<const uint2*>(orow + 64 + i0);
    }
    in.c01 = reinterpret_cast<const float4*>(rec)[i0 >> 1];  // (cos, sin) of pairs i0, i0 + 1
    in.c23 = reinterpret_cast<const float4*>(rec)[(i0 >> 1) + 1];
  };

  // ---- loads that do not depend on the sequence length go out first ------------------------
  typedef typename std::conditional<SUB == 4, uint2, uint4>::type cw_t;
  cw_t cw_reg = {};
  if (tid < kCodes) cw_reg = reinterpret_cast<const cw_t*>(codebook)[tid];
  constexpr int QPT = (4 * kHeadDim + NT - 1) / NT;  // query elements per thread
  float qv[QPT];
#pragma unroll
  for (int u = 0; u < QPT; ++u) {
    const int i = tid + u * NT, hh = i >> 7, c = i & 127;
    qv[u] = (i < 4 * kHeadDim && hh < r) ? __half2float(q[(int64_t)(b * g.n_q_heads + hq0 + hh) * kHeadDim + c]) : 0.f;
  }
  // ROPE: the fp16 cosine / sine rows go to LDS with the codebook (four 16-byte chunks per thread)
  constexpr int TROWS = ROPE ? (2048 + NT - 1) / NT : 1;  // 2048 16-byte chunks of the hi and lo rows
  uint4 trow[TROWS];
  if constexpr (ROPE) {  // (the residual wave and the last round's surplus threads load in-bounds chunks that they never store)
#pragma unroll
    for (int u = 0; u < TROWS; ++u)
      trow[u] = reinterpret_cast<const uint4*>(g.rope + kRopeHiOff)[min(min(tid, NT - 1) + u * NT, 2047)];
  }
  RopeIn rin = {};
  if constexpr (ROPE) {
    if (main_wave) rope_load(wave, rin);  // first batch: in bounds whatever the length
  }
  Grp cur;
  const bool spec = main_wave && !g.paged && (t0 + (wave << 6) + 64 <= g.page_tokens);  // in bounds whatever the length
  if (spec) load_group(wave, true, cur);
  // The split's first Shift group is shared by all waves when there is one group per sequence:
  // its q . o^k is formed once per workgroup (waves that do not rotate a query head), not per wave.
  static_assert(NW >= 8 || (ROPE && NW == 7), "prologue work split: waves 0-3 rotate the query, waves 4.. do the rest "
                                              "(waves 4..7 take a head's q . o^k unless the mean is turned in the kernel)");
  const int grp_pre = group_of(g, min(t0, g.page_tokens * g.pages_per_seq - 1));
  Side pre = {};  // only the key-side mean fields are used
  if (!ROPE && wave >= 4 && wave - 4 < R) {
    if constexpr (DQ) {
      const unsigned char* km = reinterpret_cast<const unsigned char*>(kc.means) + (mean_base + grp_pre) * kDqMeanRec;
      pre.okq = km[lane];
      pre.okp = *reinterpret_cast<const __half2*>(km + kDqMeanPar + 4 * (lane >> 4));
    } else {
      pre.ok2 = *reinterpret_cast<const __half2*>(
          reinterpret_cast<const unsigned char*>(kc.means + (mean_base + grp_pre) * kHeadDim) + lane_x4);
    }
  }
  // With several Shift groups per split (group_size > 0), wave 5 forms q . o^k of all of them at
  // once: lane j owns group g_first + j, its fp16 mean row is the B operand of the same contraction
  // that the residual tokens use (unrotated query hi + lo as the A operand), 64 MFMAs in the
  // shadow of the table fill instead of four wave-wide sums per group and wave in the main loop.
  const int g_first = grp_pre;
  int n_tab = 0;
  if (!ROPE && !DQ && g.group_size > 0) {  // (4-bit means: no fp16 rows to feed the matrix cores; in-loop form)
    const int g_last = group_of(g, min(t0 + per - 1, g.page_tokens * g.pages_per_seq - 1));
    n_tab = g_last - g_first + 1;
    if (n_tab > SM::kQoTabGroups) n_tab = 0;  // very long splits keep the in-loop form
  }
  uint4 orow[16];  // one 256-byte mean row
  const bool tab_wave = (wave == 5) && n_tab > 0;
  if (tab_wave) {
    const uint4* rp = reinterpret_cast<const uint4*>(kc.means + (mean_base + min(g_first + lane, g.n_groups_max - 1)) * kHeadDim);
#pragma unroll
    for (int u = 0; u < 16; ++u) orow[u] = (lane < n_tab) ? rp[u] : make_uint4(0u, 0u, 0u, 0u);
  }
  const int len = seq_lens[b];  // scalar load in flight; first used after the prologue

  // ---- prologue: codebook table, rotated query (independent of the sequence length) ----------
  if (tid < kCodes) reinterpret_cast<cw_t*>(sm_stage)[tid] = cw_reg;
#pragma unroll
  for (int u = 0; u < QPT; ++u) {
    const int i = tid + u * NT;
    if (i < 4 * kHeadDim) sm_q_orig[i >> 7][i & 127] = qv[u];
  }
  if constexpr (ROPE) {
    if (main_wave) {
#pragma unroll
      for (int u = 0; u < TROWS; ++u) {
        const int c = tid + u * NT;  // chunk c: part (hi / lo) c >> 10, row (c >> 4) & 63, 16-byte chunk c & 15
        const int row = (c >> 4) & 63;
        if (NT * TROWS == 2048 || c < 2048)
          *reinterpret_cast<uint4*>(sm_rope_tab + (c >> 10) * 16384 + row * 256 + (((c & 15) ^ (row & 15)) << 4)) = trow[u];
      }
    }
  }
  __syncthreads();
  const float qscale = (float)kInvSqrtD * scale_log2e;
  for (int hh = wave; hh < 4; hh += NW) {  // d1: one wave rotates one head, butterflies across lanes
    float x0 = sm_q_orig[hh][2 * lane], x1 = sm_q_orig[hh][2 * lane + 1];
    {
      const float a0 = x0 + x1, a1 = x0 - x1;
      x0 = a0, x1 = a1;
    }
    static_for<6>([&](auto kc) {  // lane bit k <-> element bit k + 1
      constexpr int m = 1 << decltype(kc)::value;
      const float p0 = xor_lane<m>(x0), p1 = xor_lane<m>(x1);
      const bool upper = (lane & m) != 0;
      x0 = upper ? p0 - x0 : x0 + p0;
      x1 = upper ? p1 - x1 : x1 + p1;
    });
    sm_q_had[hh][2 * lane] = x0 * qscale;
    sm_q_had[hh][2 * lane + 1] = x1 * qscale;
  }
  if constexpr (SGN) {
    // sign-mask table at LDS address 0: row = sign nibble n (256 bytes), 32 copies of the 8-byte entry
    // whose four fp16 sign bits are bits 0..3 of n
    for (int e = tid; e < 16 * 32; e += NT) {  // (one round with 8 waves)
      if (!main_wave) break;
      const uint32_t n = e >> 5;
      const uint32_t w0 = ((n & 1u) ? 0x8000u : 0u) | ((n & 2u) ? 0x80000000u : 0u);
      const uint32_t w1 = ((n & 4u) ? 0x8000u : 0u) | ((n & 8u) ? 0x80000000u : 0u);
      *reinterpret_cast<uint2*>(sm_table + n * 256 + (e & 31) * 8) = make_uint2(w0, w1);
    }
  }
  if (!ROPE && wave >= 4 && wave - 4 < R) {
    const int hh = wave - 4;
    float op0, op1;
    mean_pair(pre, true, op0, op1);
    const float dot = wave_sum_u(sm_q_orig[hh][2 * lane] * op0 + sm_q_orig[hh][2 * lane + 1] * op1);
    if (lane == 0) sm_qo_first[hh] = dot * scale_log2e;
  }
  if (tab_wave) {
    h4 AH[2], AL[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int row = lane & 3;
      const int head = PACK ? row % R : row;
      const bool is_lo = PACK && row >= R, dead = (PACK && row >= 2 * R) || head >= r;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float x = dead ? 0.f : sm_q_orig[head][4 * (16 * p + (lane >> 2)) + k] * scale_log2e;
        const _Float16 hi = (_Float16)x;
        const _Float16 lo = (_Float16)(x - (float)hi);
        AH[p][k] = is_lo ? lo : hi;
        AL[p][k] = lo;
      }
    }
    f4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
    static_for<16>([&](auto uc) {  // 16 bytes = slots 2u, 2u + 1 (four channels each)
      constexpr int u = decltype(uc)::value;
      const h4 b0 = as_h4(orow[u].x, orow[u].y), b1 = as_h4(orow[u].z, orow[u].w);
      d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(AH[(2 * u) / 16], b0, d0, 4, (2 * u) % 16, 0);
      d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(AH[(2 * u + 1) / 16], b1, d1, 4, (2 * u + 1) % 16, 0);
      if constexpr (!PACK) {
        d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(AL[(2 * u) / 16], b0, d0, 4, (2 * u) % 16, 0);
        d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(AL[(2 * u + 1) / 16], b1, d1, 4, (2 * u + 1) % 16, 0);
      }
    });
    float4 t4 = make_float4(0.f, 0.f, 0.f, 0.f);
    float* tv = &t4.x;
#pragma unroll
    for (int i = 0; i < R; ++i) tv[i] = PACK ? (d0[i] + d0[R + i]) + (d1[i] + d1[R + i]) : d0[i] + d1[i];
    if (lane < n_tab) sm_qo_tab[lane] = t4;
  }
  {  // replicate the staged codewords with 16-byte LDS writes (8-byte codewords go out in pairs);
    // the four waves that rotated a query head take 6 of the 16-byte slots per thread, the others 10
    constexpr int NW16 = 16;  // 16-byte slots per 256-byte code row
    typedef uint32_t u4v __attribute__((ext_vector_type(4)));
    typedef uint32_t u2v __attribute__((ext_vector_type(2)));
    auto fill = [&](auto nc, int first, auto stride_c) {
      constexpr int N = decltype(nc)::value;
      constexpr int STRIDE = decltype(stride_c)::value;
      constexpr bool GUARD = (STRIDE != 256);  // other wave counts: the last round may run past the table
      u4v tmp[N];
#pragma unroll
      for (int u = 0; u < N; ++u) {
        const int code = min((first + u * STRIDE) >> 4, kCodes - 1);
        if constexpr (SUB == 4) {
          const u2v c2 = reinterpret_cast<const u2v*>(sm_stage)[code];
          tmp[u] = u4v{c2.x, c2.y, c2.x, c2.y};
        } else {
          tmp[u] = reinterpret_cast<const u4v*>(sm_stage)[code];
        }
      }
#pragma unroll
      for (int u = 0; u < N; ++u) {
        const int i = first + u * STRIDE;
        if (!GUARD || i < kCodes * NW16)
          *reinterpret_cast<u4v*>(sm_table + TB + (i >> 4) * 256 + (i & 15) * 16) = tmp[u];
      }
    };
    if constexpr (NW == 8) {
      static_assert(256 * 6 + 256 * 10 == kCodes * NW16, "slot split must cover the table");
      if (wave < 4)
        fill(std::integral_constant<int, 6>{}, tid, std::integral_constant<int, 256>{});
      else if (main_wave)
        fill(std::integral_constant<int, 10>{}, 256 * 6 + (tid - 256), std::integral_constant<int, 256>{});
    } else {  // the four rotating waves take 4 slots per thread, the other NW - 4 waves share the rest
      constexpr int REST = (NW - 4) * 64, ROUNDS = (kCodes * NW16 - 1024 + REST - 1) / REST;
      if (wave < 4)
        fill(std::integral_constant<int, 4>{}, tid, std::integral_constant<int, 256>{});
      else if (main_wave)
        fill(std::integral_constant<int, ROUNDS>{}, 1024 + (tid - 256), std::integral_constant<int, REST>{});
    }
  }
  __syncthreads();
  const int t1 = min(len, t0 + per);
  const int n_grp = (main_wave && t1 > t0) ? (t1 - t0 + 63) >> 6 : 0;  // the residual wave owns no coded group
  if (!spec && wave < n_grp) load_group(wave, true, cur);

  // A operands of the score contraction: slot s = channels [4s, 4s+4); block (lane / 4) of
  // register pair p holds slot 16 p + block for head (lane % 4); fp16 hi and lo parts.
  h4 QH[2], QL[2];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int row = lane & 3;
    const int head = PACK ? row % R : row;          // PACK: rows [0,R) hi, [R,2R) lo, rest zero
    const bool is_lo = PACK && row >= R, dead = PACK && row >= 2 * R;
    const float* src = &sm_q_had[head][4 * (16 * p + (lane >> 2))];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float x = src[k];
      const _Float16 hi = (_Float16)x;
      const _Float16 lo = (_Float16)(x - (float)hi);
      QH[p][k] = dead ? (_Float16)0.f : (is_lo ? lo : hi);
      QL[p][k] = lo;
    }
  }
  float qo_pre[4];  // wave-uniform: lives in scalar registers
#pragma unroll
  for (int i = 0; i < 4; ++i)
    qo_pre[i] = __builtin_bit_cast(
        float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sm_qo_first[i < R ? i : 0])));
  const uint32_t laneoff = (SUB == 4) ? (lane & 31) * 8 : (lane & 15) * 16;
  const uint32_t laneoff8 = (lane & 31) * 8;  // sign-mask table: 32 copies of 8 bytes per 256-byte row
#pragma unroll
  for (int i = 0; i < 4; ++i)  // wave-private; every lane owns channels 2 lane, 2 lane + 1 of each head
    *reinterpret_cast<float2*>(&sm_accm[wave][i][2 * lane]) = make_float2(0.f, 0.f);

  float m_run[4], l_run[4], beta[4], cf[4], qo[4];  // entries [0,R) are live
  f4 acc[SUB];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m_run[i] = -INFINITY;
    l_run[i] = 0.f;
    beta[i] = 0.f;
    cf[i] = 1.f;
    qo[i] = 0.f;
  }
#pragma unroll
  for (int c = 0; c < SUB; ++c) acc[c] = f4{0.f, 0.f, 0.f, 0.f};
  int cur_group = -1;
  float ov0 = 0.f, ov1 = 0.f;  // this lane's two channels of the current group's o^v

  // mean-vector term of the Shift group that just ended: accm = accm * cf + (sum of beta) * o^v
  auto flush_group = [&]() {
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const float bsum = wave_sum_u(beta[i]);
      float* dst = &sm_accm[wave][i][2 * lane];
      dst[0] = dst[0] * cf[i] + bsum * ov0;
      dst[1] = dst[1] * cf[i] + bsum * ov1;
      beta[i] = 0.f;
      cf[i] = 1.f;
    }
  };

  // sign format: the two 8-byte mask entries (low nibble -> channels 0..3, high nibble -> 4..7)
  // of sign byte k of `sw`; each mask word carries the fp16 sign bits of two channels
  constexpr int MB = SGN ? CH : 1;  // mask buffers exist only in the sign format
  auto sign_masks = [&](uint32_t sw, int k) -> uint4 {
    const uint32_t p8 = perm_b32(sw, laneoff8, 0x0c0c0400u + (k << 8));  // (sign byte << 8) | lane offset
    const uint2 lo = lds_read64(p8 & 0x0FFFu);
    const uint2 hi = lds_read64(((p8 >> 4) & 0x0F00u) | laneoff8);
    return make_uint4(lo.x, lo.y, hi.x, hi.y);
  };
  auto k_gather = [&](const uint32_t (&kcode)[KW], auto cc, cw_t (&buf)[CH], uint4 (&mb)[MB]) {
    constexpr int ch = decltype(cc)::value;
#pragma unroll
    for (int e = 0; e < CH; ++e) {
      const int sv = CH * ch + e;  // sub-vector: byte sv % 4 of index dword sv / 4
      const uint32_t addr = perm_b32(kcode[sv / 4], laneoff, 0x0c0c0400u + ((sv % 4) << 8));
      if constexpr (SUB == 4)
        buf[e] = lds_read64(addr);
      else
        buf[e] = lds_read128(addr + TB);
      if constexpr (SGN) mb[e] = sign_masks(kcode[IW + sv / 4], sv % 4);
    }
  };
  auto k_contract = [&](auto cc, auto signed_c, const cw_t (&buf)[CH], const uint4 (&mb)[MB], const h4 (&QH)[2],
                        const h4 (&QL)[2], f4& d0, f4& d1) {
    constexpr int ch = decltype(cc)::value;
    constexpr bool apply_sign = decltype(signed_c)::value;
    static_for<CH>([&](auto ec) {
      constexpr int e = decltype(ec)::value;
      constexpr int s = CH * ch + e;
      if constexpr (SUB == 4) {
        const h4 bop = as_h4(buf[e].x, buf[e].y);
        d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(QH[s / 16], bop, d0, 4, s % 16, 0);
        if constexpr (!PACK) d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(QL[s / 16], bop, d1, 4, s % 16, 0);
      } else {
        uint4 c = make_uint4(buf[e].x, buf[e].y, buf[e].z, buf[e].w);
        if constexpr (apply_sign) c = make_uint4(c.x ^ mb[e].x, c.y ^ mb[e].y, c.z ^ mb[e].z, c.w ^ mb[e].w);
        const h4 b0 = as_h4(c.x, c.y), b1 = as_h4(c.z, c.w);
        d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(QH[(2 * s) / 16], b0, d0, 4, (2 * s) % 16, 0);
        d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(QH[(2 * s + 1) / 16], b1, d1, 4, (2 * s + 1) % 16, 0);
        if constexpr (!PACK) {
          d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(QL[(2 * s) / 16], b0, d0, 4, (2 * s) % 16, 0);
          d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(QL[(2 * s + 1) / 16], b1, d1, 4, (2 * s + 1) % 16, 0);
        }
      }
    });
  };
  constexpr int VMB = SGN ? 4 : 1;
  auto v_gather = [&](uint32_t vw, uint32_t sw, cw_t (&buf)[4], uint4 (&mb)[VMB]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t addr = perm_b32(vw, laneoff, 0x0c0c0400u + (k << 8));
      if constexpr (SUB == 4)
        buf[k] = lds_read64(addr);
      else
        buf[k] = lds_read128(addr + TB);
      if constexpr (SGN) mb[k] = sign_masks(sw, k);
    }
  };
  auto v_contract = [&](auto ac, auto signed_c, const cw_t (&cw)[4], const uint4 (&mb)[VMB], const h4& wop,
                        f4 (&acc)[SUB]) {
    constexpr int a = decltype(ac)::value;
    constexpr bool apply_sign = decltype(signed_c)::value;
    if constexpr (SUB == 4) {
      const h4 b0 = as_h4(perm_b32(cw[1].x, cw[0].x, 0x05040100u), perm_b32(cw[3].x, cw[2].x, 0x05040100u));
      const h4 b1 = as_h4(perm_b32(cw[1].x, cw[0].x, 0x07060302u), perm_b32(cw[3].x, cw[2].x, 0x07060302u));
      const h4 b2 = as_h4(perm_b32(cw[1].y, cw[0].y, 0x05040100u), perm_b32(cw[3].y, cw[2].y, 0x05040100u));
      const h4 b3 = as_h4(perm_b32(cw[1].y, cw[0].y, 0x07060302u), perm_b32(cw[3].y, cw[2].y, 0x07060302u));
      acc[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b0, acc[0], CBSZ_V, a, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b1, acc[1], CBSZ_V, a, 0);
      acc[2] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b2, acc[2], CBSZ_V, a, 0);
      acc[3] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b3, acc[3], CBSZ_V, a, 0);
    } else {
      uint32_t c0[4] = {cw[0].x, cw[0].y, cw[0].z, cw[0].w};
      uint32_t c1[4] = {cw[1].x, cw[1].y, cw[1].z, cw[1].w};
      uint32_t c2[4] = {cw[2].x, cw[2].y, cw[2].z, cw[2].w};
      uint32_t c3[4] = {cw[3].x, cw[3].y, cw[3].z, cw[3].w};
      if constexpr (apply_sign) {
        c0[0] ^= mb[0].x, c0[1] ^= mb[0].y, c0[2] ^= mb[0].z, c0[3] ^= mb[0].w;
        c1[0] ^= mb[1].x, c1[1] ^= mb[1].y, c1[2] ^= mb[1].z, c1[3] ^= mb[1].w;
        c2[0] ^= mb[2].x, c2[1] ^= mb[2].y, c2[2] ^= mb[2].z, c2[3] ^= mb[2].w;
        c3[0] ^= mb[3].x, c3[1] ^= mb[3].y, c3[2] ^= mb[3].z, c3[3] ^= mb[3].w;
      }
      static_for<4>([&](auto mc) {
        constexpr int mth = decltype(mc)::value;
        const h4 be = as_h4(perm_b32(c1[mth], c0[mth], 0x05040100u), perm_b32(c3[mth], c2[mth], 0x05040100u));
        const h4 bo = as_h4(perm_b32(c1[mth], c0[mth], 0x07060302u), perm_b32(c3[mth], c2[mth], 0x07060302u));
        acc[2 * mth] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, be, acc[2 * mth], CBSZ_V, a, 0);
        acc[2 * mth + 1] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, bo, acc[2 * mth + 1], CBSZ_V, a, 0);
      });
    }
  };

  // d3/d4: scores in log2 units, lazy running max, weights.  Returns the fp16 weights as the
  // value-side A operand: lane i of a quad holds head i, the quad's four tokens.
  float a_run = 0.f, w_scale = 0.f;  // A (0 = no token yet) and 2^10 / A, the same in every lane
  auto softmax_step = [&](const f4& d0, const f4& d1, bool valid, float a_k, float b_k, float a_v, float b_v) -> h4 {
    float s[4], w[4];
    bool need = a_v > a_run;
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const float dot = PACK ? (d0[i] + d0[R + i]) + (d1[i] + d1[R + i]) : d0[i] + d1[i];
      s[i] = valid ? fmaf(a_k, dot, b_k * qo[i]) : -INFINITY;
      need = need || (s[i] - m_run[i] > kLazyMaxLog2);
    }
    if (__any(need)) {
      // A: the next power of two >= the largest a^v of the wave (kept once it is large enough)
      const float amax_w = wave_max_u(a_v);
      float a_new = a_run;
      if (amax_w > a_run) a_new = __uint_as_float((__float_as_uint(amax_w) + 0x007fffffu) & 0x7f800000u);
      const float a_inv = (a_new > 0.f) ? __builtin_amdgcn_rcpf(a_new) : 0.f;  // exact: a power of two
      const float a_ratio = a_run * a_inv;
      a_run = a_new;
      w_scale = kWeightScaleM * a_inv;
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const float m_new = fmaxf(m_run[i], wave_max_u(s[i]));
        const float corr = (m_run[i] == -INFINITY) ? 0.f : fast_exp2(m_run[i] - m_new);
        l_run[i] *= corr;
        beta[i] *= corr;
        cf[i] *= corr;
        const float corr_a = corr * a_ratio;
#pragma unroll
        for (int c = 0; c < SUB; ++c) acc[c][i] *= corr_a;
        m_run[i] = m_new;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = 0.f;
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const float p = fast_exp2(s[i] - m_run[i]);  // 0 for masked lanes
      l_run[i] += p;
      beta[i] = fmaf(p, b_v, beta[i]);
      w[i] = p * (a_v * w_scale);
    }
    quad_transpose(w, lane);
    h4 wop;
#pragma unroll
    for (int k = 0; k < 4; ++k) wop[k] = (_Float16)w[k];
    return wop;
  };

  // ROPE: q . RoPE_t(o^k) (log2 units) for the 64 tokens of this wave's groups gi0, gi0 + NW, ... (four of
  // them): lane (m = lane % 16, kq = lane / 16) supplies row (group m / 4, head m % 4) of the turned
  // products A', B' at channels 32 ks + 8 kq + e and column m of the token-side table.
  auto rope_compute = [&](const RopeIn& in) {
    const int m = lane & 15, head = m & 3, kq = lane >> 4;
    // the block's turned mean ro = RoPE_(64 block)(o) (times the score scale) at this lane's four pairs;
    // with it  A'_i = q_i ro_i + q_i' ro_i',  B'_i = q_i' ro_i - q_i ro_i'
    float rl[4], rh[4];
    {
      const h4 oa = as_h4(in.oa.x, in.oa.y), ob = as_h4(in.ob.x, in.ob.y);
      const float cs[8] = {in.c01.x, in.c01.y, in.c01.z, in.c01.w, in.c23.x, in.c23.y, in.c23.z, in.c23.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float o0 = DQ ? lvl(in.oap, (in.oaq >> (4 * e)) & 15u) : (float)oa[e];
        const float o1 = DQ ? lvl(in.obp, (in.obq >> (4 * e)) & 15u) : (float)ob[e];
        const float cc = cs[2 * e] * scale_log2e, ss = cs[2 * e + 1] * scale_log2e;
        rl[e] = o0 * cc - o1 * ss;
        rh[e] = o1 * cc + o0 * ss;
      }
    }
    h8d AH[4], AL[4];
    static_for<4>([&](auto cc) {  // chunk c of the quad's lane c: four pairs from i0
      constexpr int c = decltype(cc)::value;
      constexpr int ksp = c >> 1, hf = c & 1;
      constexpr int ctrl = c | (c << 2) | (c << 4) | (c << 6);  // quad_perm: every lane reads lane c of its quad
      const int i0 = 32 * ksp + 8 * kq + 4 * hf;
      const float4 a4 = *reinterpret_cast<const float4*>(&sm_q_keep[head][i0]);
      const float4 b4 = *reinterpret_cast<const float4*>(&sm_q_keep[head][64 + i0]);
      const float qa[4] = {a4.x, a4.y, a4.z, a4.w}, qb[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float xl = dpp_quad<ctrl>(rl[e]), xh = dpp_quad<ctrl>(rh[e]);
        const float Ap = qa[e] * xl + qb[e] * xh, Bp = qb[e] * xl - qa[e] * xh;
        const _Float16 ah = (_Float16)Ap, bh = (_Float16)Bp;
        AH[ksp][4 * hf + e] = ah;
        AL[ksp][4 * hf + e] = (_Float16)(Ap - (float)ah);
        AH[ksp + 2][4 * hf + e] = bh;
        AL[ksp + 2][4 * hf + e] = (_Float16)(Bp - (float)bh);
      }
    });
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
      f4 d = {0.f, 0.f, 0.f, 0.f};
      const uint32_t row_addr = SM::kRopeTabOffset + (16 * tile + m) * 256;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint32_t a = row_addr + (((4 * ks + kq) ^ m) << 4);
        const h8d th = __builtin_bit_cast(h8d, lds_read128(a));
        const h8d tl = __builtin_bit_cast(h8d, lds_read128(a + 16384));
        d = __builtin_amdgcn_mfma_f32_16x16x32_f16(AH[ks], th, d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_16x16x32_f16(AL[ks], th, d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_16x16x32_f16(AH[ks], tl, d, 0, 0, 0);
      }
      // this lane holds group kq, token 16 tile + m, heads 0..3
      sm_rope_dot[wave][kq][16 * tile + m] = make_float4(d[0], d[1], d[2], d[3]);
    }
    // the entries are read back by other lanes of this wave
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };

  // the first batch (groups wave, wave + NW, ...) from the operands loaded at kernel start
  if constexpr (ROPE) {
    if (n_grp > wave) rope_compute(rin);
  }

  // ---- main loop: this wave's 64-token groups, next group's loads in flight ------------------
  int it = 0;  // this wave's iteration count
  for (int gi = wave; gi < n_grp; gi += NW, ++it) {
    const int tg = t0 + (gi << 6);  // first token of the group (multiple of 64)
    const bool valid = (tg + lane) < t1;
    const bool has_next = gi + NW < n_grp;  // wave-uniform
    constexpr bool kInPlace = SGN;
    if constexpr (ROPE) {  // before the next group's loads are issued: fewer live registers
      if (it > 0 && (it & (SM::kRopeBatch - 1)) == 0) {
        RopeIn in;
        rope_load(gi, in);
        rope_compute(in);
      }
    }
    Side nxt;
    Grp nxt_full;
    if constexpr (kInPlace)
      load_side(gi + NW, has_next, nxt);
    else
      load_group(gi + NW, has_next, nxt_full);
    // (selects, not a branch on `valid`: a branch would pin the wait for these registers to the top of
    // the iteration, right behind the next group's loads)
    float a_k, b_k, a_v, b_v;
    if constexpr (DQ) {  // b = min + step * code, a = b * a'
      const uint32_t sh = (lane & 1) * 4;
      const float bk = lvl(cur.s.kp, (cur.s.kq >> sh) & 15u), bv = lvl(cur.s.vp, (cur.s.vq >> sh) & 15u);
      a_k = valid ? bk * half_bits(cur.s.ka) : 0.f, b_k = valid ? bk : 0.f;
      a_v = valid ? bv * half_bits(cur.s.va) : 0.f, b_v = valid ? bv : 0.f;
    } else {
      a_k = valid ? __low2float(cur.s.nk) : 0.f, b_k = valid ? __high2float(cur.s.nk) : 0.f;
      a_v = valid ? __low2float(cur.s.nv) : 0.f, b_v = valid ? __high2float(cur.s.nv) : 0.f;
    }

    // Shift group bookkeeping (wave-uniform): mean term of the old group, q . o^k of the new one
    const int grp = group_of(g, tg);
    if constexpr (ROPE) {  // this token's q . RoPE_t(o^k), four heads
      const float4 rd = sm_rope_dot[wave][it & (SM::kRopeBatch - 1)][lane];
      const float rv[4] = {rd.x, rd.y, rd.z, rd.w};
#pragma unroll
      for (int i = 0; i < R; ++i) qo[i] = rv[i];
    }
    if (grp != cur_group) {
      if (cur_group >= 0) flush_group();
      if constexpr (ROPE) {
        // the mean term is per token (above)
      } else if (grp - g_first < n_tab) {  // n_tab > 0 only with group_size > 0
        const float4 t4 = sm_qo_tab[grp - g_first];
        const float tv[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
        for (int i = 0; i < R; ++i) qo[i] = tv[i];
      } else if (grp == grp_pre) {
#pragma unroll
        for (int i = 0; i < R; ++i) qo[i] = qo_pre[i];
      } else {
        float o0, o1;
        mean_pair(cur.s, true, o0, o1);
#pragma unroll
        for (int i = 0; i < R; ++i) {
          const float2 q2 = *reinterpret_cast<const float2*>(&sm_q_keep[i][2 * lane]);
          qo[i] = wave_sum_u(q2.x * o0 + q2.y * o1) * scale_log2e;
        }
      }
      mean_pair(cur.s, false, ov0, ov1);
      cur_group = grp;
    }

    // d2/d3: HT(q) . C[codes] for four heads; gathers of chunk c+1 are issued before the
    // contractions of chunk c
    f4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
    {
      cw_t bufA[CH], bufB[CH];
      uint4 mskA[MB], mskB[MB];
      constexpr std::integral_constant<bool, SGN> sgn{};
      k_gather(cur.kcode, std::integral_constant<int, 0>{}, bufA, mskA);
      static_for<NSV / CH>([&](auto cc) {
        constexpr int ch = decltype(cc)::value;
        if constexpr (ch % 2 == 0) {
          if constexpr (ch + 1 < NSV / CH) k_gather(cur.kcode, std::integral_constant<int, ch + 1>{}, bufB, mskB);
          k_contract(cc, sgn, bufA, mskA, QH, QL, d0, d1);
        } else {
          if constexpr (ch + 1 < NSV / CH) k_gather(cur.kcode, std::integral_constant<int, ch + 1>{}, bufA, mskA);
          k_contract(cc, sgn, bufB, mskB, QH, QL, d0, d1);
        }
      });
    }
    if constexpr (kInPlace)
      load_k_codes(gi + NW, has_next, cur);  // the key codes are consumed: refill them in place
    constexpr std::integral_constant<bool, SGN> vsgn{};
    cw_t vbufA[4], vbufB[4];
    uint4 vmskA[VMB], vmskB[VMB];
    // first value-side gathers fly during the softmax arithmetic
    v_gather(cur.vcode[0], cur.vcode[SGN ? IW : 0], vbufA, vmskA);

    const h4 wop = softmax_step(d0, d1, valid, a_k, b_k, a_v, b_v);

    // d5: out_rot[head][channel] += sum over tokens of weight * codeword channel
    static_for<IW>([&](auto ac) {
      constexpr int a = decltype(ac)::value;
      constexpr int sa = SGN ? IW + a + 1 : 0;  // dword of the next round's sign bytes
      if constexpr (SGN) {  // one buffer (32 registers with its masks): gather the next round after this one's MFMAs
        v_contract(ac, vsgn, vbufA, vmskA, wop, acc);
        if constexpr (a + 1 < IW) v_gather(cur.vcode[a + 1], cur.vcode[sa], vbufA, vmskA);
      } else if constexpr (a % 2 == 0) {
        if constexpr (a + 1 < IW) v_gather(cur.vcode[a + 1], cur.vcode[sa], vbufB, vmskB);
        v_contract(ac, vsgn, vbufA, vmskA, wop, acc);
      } else {
        if constexpr (a + 1 < IW) v_gather(cur.vcode[a + 1], cur.vcode[sa], vbufA, vmskA);
        v_contract(ac, vsgn, vbufB, vmskB, wop, acc);
      }
    });
    if constexpr (kInPlace) {
      load_v_codes(gi + NW, has_next, cur);  // likewise the value codes
      cur.s = nxt;
    } else {
      cur = nxt_full;
    }
  }

  // ---- residual (Sec. 3.2): the most recent tokens are still fp16 and join the same softmax ---
  // The extra wave of the last split treats them as one more 64-token group: the fp16 key row of
  // the lane's token is the B operand directly (no table), the A operand is the unrotated query,
  // and the value rows accumulate in the original domain next to the mean-vector term.
  f4 acc_res[SUB];
  bool res_here = false;
  if (res.k != nullptr && split == n_splits - 1 && wave == NW) {
    const int rl = min(res.lens[b], res.capacity);
    if (rl > 0) {
      res_here = true;
      const bool valid = lane < rl;
      h4 AH[2], AL[2];
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        const int row = lane & 3;
        const int head = PACK ? row % R : row;
        const bool is_lo = PACK && row >= R, dead = (PACK && row >= 2 * R) || head >= r;
        uint2 raw = make_uint2(0u, 0u);
        if (!dead)
          raw = *reinterpret_cast<const uint2*>(q + (int64_t)(b * g.n_q_heads + hq0 + head) * kHeadDim +
                                                4 * (16 * p + (lane >> 2)));
        const h4 qh = as_h4(raw.x, raw.y);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float x = (float)qh[k] * scale_log2e;
          const _Float16 hi = (_Float16)x;
          const _Float16 lo = (_Float16)(x - (float)hi);
          AH[p][k] = is_lo ? lo : hi;
          AL[p][k] = lo;
        }
      }
      const int64_t unit_row = (int64_t)(b * g.n_kv_heads + h) * res.capacity;
      f4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
      const uint4 no_mask[MB] = {};
      const uint4 no_vmask[VMB] = {};
      constexpr std::false_type plain{};  // fp16 rows carry their own signs
      if constexpr (SM::kResInLds) {
        // A lane needs its own token's whole key row, 8 or 16 bytes per MFMA: read straight from global
        // memory that is 64 different cache lines per load instruction (measured +1.3 us per launch with a
        // full residual).  Instead the rows come in with coalesced loads (an instruction covers four
        // consecutive rows), go to LDS, and every lane reads its row from there; rows past the valid
        // count are stored as zeros.
        const uint32_t sk = SM::kResOffset, sv = SM::kResOffset + 64 * SM::kResKStride;
        const int sub_row = lane >> 4, piece = lane & 15;  // 16 lanes x 16 bytes = one 256-byte row
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          uint4 kx[8], vx[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int row = 4 * (8 * hf + u) + sub_row;
            kx[u] = vx[u] = make_uint4(0u, 0u, 0u, 0u);
            if (row < rl) {
              kx[u] = *reinterpret_cast<const uint4*>(res.k + (unit_row + row) * kHeadDim + piece * 8);
              vx[u] = *reinterpret_cast<const uint4*>(res.v + (unit_row + row) * kHeadDim + piece * 8);
            }
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int row = 4 * (8 * hf + u) + sub_row;
            unsigned char* kd = smem_raw + sk + row * SM::kResKStride + piece * 16;
            if constexpr (SM::kResKStride % 16 == 0) {
              *reinterpret_cast<uint4*>(kd) = kx[u];
            } else {
              *reinterpret_cast<uint2*>(kd) = make_uint2(kx[u].x, kx[u].y);
              *reinterpret_cast<uint2*>(kd + 8) = make_uint2(kx[u].z, kx[u].w);
            }
            *reinterpret_cast<uint4*>(smem_raw + sv + row * 256 + piece * 16) = vx[u];
          }
        }
        // written and read by different lanes of this one wave
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint32_t krow = sk + lane * SM::kResKStride;
        static_for<NSV / CH>([&](auto cc) {
          constexpr int ch = decltype(cc)::value;
          cw_t buf[CH];
#pragma unroll
          for (int u = 0; u < CH; ++u) {
            if constexpr (SUB == 4)
              buf[u] = lds_read64(krow + (CH * ch + u) * 8);
            else
              buf[u] = lds_read128(krow + (CH * ch + u) * 16);
          }
          k_contract(cc, plain, buf, no_mask, AH, AL, d0, d1);
        });
        const h4 wop = softmax_step(d0, d1, valid, 1.f, 0.f, 1.f, 0.f);
#pragma unroll
        for (int c = 0; c < SUB; ++c) acc_res[c] = f4{0.f, 0.f, 0.f, 0.f};
        static_for<IW>([&](auto ac) {
          constexpr int a = decltype(ac)::value;
          cw_t cw[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int t = (lane / LV) * NSV + 4 * a + k;  // the same token order as a coded group
            if constexpr (SUB == 4)
              cw[k] = lds_read64(sv + t * 256 + (lane % LV) * 8);
            else
              cw[k] = lds_read128(sv + t * 256 + (lane % LV) * 16);
          }
          v_contract(ac, plain, cw, no_vmask, wop, acc_res);
        });
      } else {
        const uint4* krow = reinterpret_cast<const uint4*>(res.k + (unit_row + lane) * kHeadDim);
        static_for<NSV / CH>([&](auto cc) {
          constexpr int ch = decltype(cc)::value;
          cw_t buf[CH];
          if constexpr (SUB == 4) {
#pragma unroll
            for (int u = 0; u < CH / 2; ++u) {
              const uint4 x = valid ? krow[(CH / 2) * ch + u] : make_uint4(0u, 0u, 0u, 0u);
              buf[2 * u] = make_uint2(x.x, x.y);
              buf[2 * u + 1] = make_uint2(x.z, x.w);
            }
          } else {
#pragma unroll
            for (int u = 0; u < CH; ++u) buf[u] = valid ? krow[CH * ch + u] : make_uint4(0u, 0u, 0u, 0u);
          }
          k_contract(cc, plain, buf, no_mask, AH, AL, d0, d1);
        });
        const h4 wop = softmax_step(d0, d1, valid, 1.f, 0.f, 1.f, 0.f);
#pragma unroll
        for (int c = 0; c < SUB; ++c) acc_res[c] = f4{0.f, 0.f, 0.f, 0.f};
        static_for<IW>([&](auto ac) {
          constexpr int a = decltype(ac)::value;
          cw_t cw[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int t = (lane / LV) * NSV + 4 * a + k;  // the same token order as a coded group
            cw[k] = cw_t{};
            if (t < rl) cw[k] = *reinterpret_cast<const cw_t*>(res.v + (unit_row + t) * kHeadDim + (lane % LV) * SUB);
          }
          v_contract(ac, plain, cw, no_vmask, wop, acc_res);
        });
      }
    }
  }
  if (cur_group >= 0) flush_group();
  if (res_here) {  // fold the residual's value sum into this wave's original-domain accumulator
    // the token parts are summed across lanes first, so that every LDS word has one writer
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
      for (int c = 0; c < SUB; ++c) {
        float v = acc_res[c][i] * (a_run * (1.0f / kWeightScaleM));
        v += xor_lane<32>(v);
        if constexpr (NPART == 4) v += xor_lane<16>(v);
        if (lane < LV) sm_accm[wave][i][lane * SUB + c] += v;
      }
  }

  // ---- epilogue: wave results -> LDS (reusing the table), merge the waves -------------------
#pragma unroll
  for (int i = 0; i < R; ++i) l_run[i] = wave_sum_u(l_run[i]);
  __syncthreads();  // every wave is done gathering from the table
  float* racc = reinterpret_cast<float*>(sm_table);  // [NW][NPART][4][128]; the tail follows it
  if (main_wave) {  // the residual wave has no rotated-domain sum
    const float acc_unit = a_run * (1.0f / kWeightScaleM);
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
      for (int c4 = 0; c4 < SUB / 4; ++c4)
        *reinterpret_cast<float4*>(&racc[((wave * NPART + lane / LV) * 4 + i) * kHeadDim + (lane % LV) * SUB + 4 * c4]) =
            make_float4(acc[4 * c4][i] * acc_unit, acc[4 * c4 + 1][i] * acc_unit, acc[4 * c4 + 2][i] * acc_unit,
                        acc[4 * c4 + 3][i] * acc_unit);
  }
#pragma unroll
  for (int i = 0; i < R; ++i)
    if (lane == i) {
      sm_wave_m[wave][i] = m_run[i];
      sm_wave_l[wave][i] = l_run[i];
    }
  __syncthreads();
  float* P = partial + ((int64_t)(b * g.n_q_heads + hq0) * n_splits + split) * kPartialStrideM;
  for (int i = tid; i < r * kHeadDim; i += NT) {
    const int hh = i >> 7, c = i & 127;
    // all LDS reads go out before the first use (fixed trip counts, the residual wave's slot
    // predicated), instead of one dependent read per wave
    float mw[NW + 1], lw[NW + 1], part[NW + 1], mean[NW + 1];
#pragma unroll
    for (int wv = 0; wv <= NW; ++wv) {
      const bool present = wv < n_waves;  // uniform: slot NW exists in residual launches only
      mw[wv] = present ? sm_wave_m[wv][hh] : -INFINITY;
      lw[wv] = present ? sm_wave_l[wv][hh] : 0.f;
      mean[wv] = present ? sm_accm[wv][hh][c] : 0.f;
      part[wv] = 0.f;
      if (wv < NW) {
#pragma unroll
        for (int pt = 0; pt < NPART; ++pt) part[wv] += racc[((wv * NPART + pt) * 4 + hh) * kHeadDim + c];
      }
    }
    float M = -INFINITY;
#pragma unroll
    for (int wv = 0; wv <= NW; ++wv) M = fmaxf(M, mw[wv]);
    float L = 0.f, orot = 0.f, omean = 0.f;
#pragma unroll
    for (int wv = 0; wv <= NW; ++wv) {
      const float e = (mw[wv] == -INFINITY) ? 0.f : fast_exp2(mw[wv] - M);
      L = fmaf(e, lw[wv], L);
      orot = fmaf(e, part[wv], orot);
      omean = fmaf(e, mean[wv], omean);
    }
    float* Ph = P + (int64_t)hh * n_splits * kPartialStrideM;
    st_agent(Ph + c, orot);
    st_agent(Ph + kHeadDim + c, omean);
    if (c == 0) {
      st_agent(Ph + 2 * kHeadDim, M);
      st_agent(Ph + 2 * kHeadDim + 1, L);
    }
  }

  // ---- d6: the last workgroup of this (sequence, kv head) merges the splits -----------------
  // The partials are published with device-scope (write-through) stores and read back with
  // device-scope loads, ordered by the arrival counter; no bulk cache write-back is needed.  The counter
  // update is relaxed on purpose: agent-scope release / acquire fences around it, which would express the
  // same order in the memory model, are compiled to a write-back of the whole L2 before and an invalidate
  // after the atomic (measured: 7 us + 4 us per launch on the 8 x 8192-token shape), and the device-scope
  // accesses do not pass through the per-XCD L2 in the first place: every wave waits for the
  // acknowledgement of its own stores (s_waitcnt 0) before the workgroup barrier that precedes the atomic.
  __builtin_amdgcn_s_waitcnt(0);  // this wave's partial stores have completed
  __syncthreads();
  if (tid == 0) {
    int* cnt = counters + (b * g.n_kv_heads + h) * kCounterStrideInts;
    const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == n_splits - 1);
    if (last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
    *sm_is_last = last;
  }
  __syncthreads();
  if (!*sm_is_last) return;
  // One wave per query head: a lane owns channels 2 lane and 2 lane + 1, merges them over the
  // splits, and the inverse Hadamard (H is its own inverse) runs across the wave's lanes in
  // registers - no LDS, no barriers.
  if (wave >= r) return;
  const int hh = wave;
  const float* Ph = partial + ((int64_t)(b * g.n_q_heads + hq0 + hh) * n_splits) * kPartialStrideM;
  auto ld2 = [](const float* p) -> float2 {  // 8-byte device-scope load (p is 8-byte aligned)
    const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32)));
  };
  float L = 0.f, x0 = 0.f, x1 = 0.f, mm0 = 0.f, mm1 = 0.f;
  constexpr int SFAST = 8;
  if (n_splits <= SFAST) {
    // few splits: every load is issued before the first use, one memory round trip in all
    float2 pml[SFAST], pr[SFAST], pq[SFAST];
#pragma unroll
    for (int s = 0; s < SFAST; ++s) {
      pml[s] = make_float2(-INFINITY, 0.f);
      pr[s] = pq[s] = make_float2(0.f, 0.f);
      if (s < n_splits) {  // uniform
        const float* ps = Ph + s * kPartialStrideM;
        pml[s] = ld2(ps + 2 * kHeadDim);
        pr[s] = ld2(ps + 2 * lane);
        pq[s] = ld2(ps + kHeadDim + 2 * lane);
      }
    }
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < SFAST; ++s) M = fmaxf(M, pml[s].x);
    if (M > -INFINITY) {
#pragma unroll
      for (int s = 0; s < SFAST; ++s) {
        const float e = s < n_splits ? fast_exp2(pml[s].x - M) : 0.f;
        L = fmaf(e, pml[s].y, L);
        x0 = fmaf(e, pr[s].x, x0);
        x1 = fmaf(e, pr[s].y, x1);
        mm0 = fmaf(e, pq[s].x, mm0);
        mm1 = fmaf(e, pq[s].y, mm1);
      }
    }
  } else {
    // many splits: chunks of SFAST with every load of a chunk issued before its first use (one memory round
    // trip per chunk instead of one per split), running max carried across the chunks
    float M = -INFINITY;
    for (int s0 = 0; s0 < n_splits; s0 += SFAST) {
      float2 pml[SFAST], pr[SFAST], pq[SFAST];
#pragma unroll
      for (int s = 0; s < SFAST; ++s) {
        pml[s] = make_float2(-INFINITY, 0.f);
        pr[s] = pq[s] = make_float2(0.f, 0.f);
        if (s0 + s < n_splits) {  // uniform
          const float* ps = Ph + (s0 + s) * kPartialStrideM;
          pml[s] = ld2(ps + 2 * kHeadDim);
          pr[s] = ld2(ps + 2 * lane);
          pq[s] = ld2(ps + kHeadDim + 2 * lane);
        }
      }
      float Mn = M;
#pragma unroll
      for (int s = 0; s < SFAST; ++s) Mn = fmaxf(Mn, pml[s].x);
      if (Mn > -INFINITY) {
        const float corr = (M == -INFINITY) ? 0.f : fast_exp2(M - Mn);
        L *= corr, x0 *= corr, x1 *= corr, mm0 *= corr, mm1 *= corr;
#pragma unroll
        for (int s = 0; s < SFAST; ++s) {
          const float e = (s0 + s < n_splits) ? fast_exp2(pml[s].x - Mn) : 0.f;  // 2^-inf = 0 for empty splits
          L = fmaf(e, pml[s].y, L);
          x0 = fmaf(e, pr[s].x, x0);
          x1 = fmaf(e, pr[s].y, x1);
          mm0 = fmaf(e, pq[s].x, mm0);
          mm1 = fmaf(e, pq[s].y, mm1);
        }
        M = Mn;
      }
    }
  }
  {
    const float a0 = x0 + x1, a1 = x0 - x1;
    x0 = a0, x1 = a1;
  }
  static_for<6>([&](auto kc) {  // lane bit k <-> element bit k + 1
    constexpr int m = 1 << decltype(kc)::value;
    const float p0 = xor_lane<m>(x0), p1 = xor_lane<m>(x1);
    const bool upper = (lane & m) != 0;
    x0 = upper ? p0 - x0 : x0 + p0;
    x1 = upper ? p1 - x1 : x1 + p1;
  });
  float2 o2 = make_float2(0.f, 0.f);
  if (L > 0.f) o2 = make_float2((x0 * (float)kInvSqrtD + mm0) / L, (x1 * (float)kInvSqrtD + mm1) / L);
  *reinterpret_cast<float2*>(out + (int64_t)(b * g.n_q_heads + hq0 + hh) * kHeadDim + 2 * lane) = o2;
}

// ---------------------------------------------------------------------------------------
template <int SUB, int NW, int R, bool SGN = false, bool ROPE = false, bool DQ = false>
static int launch_one(const Geometry& g, const void* codebook, const void* q, const CacheView& kv,
                      const CacheView& vv, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                      int n_splits, void* workspace, size_t counter_bytes, const ResidualView& res, int head_off,
                      int r_pass, float* out, hipStream_t stream) {
  using SM = DecSmem<SUB, NW, SGN, ROPE>;
  const size_t smem_max = SM::kResOffset + SM::kResBytes;  // residual launches stage the fp16 rows behind the rest
  const size_t smem = res.k != nullptr ? smem_max : (size_t)SM::kBytes;
  // once per instance (thread-safe static initialisation): the gathers address the codebook table by
  // absolute LDS address, so it must start at 0, i.e. the kernel may not own any static LDS in front of
  // its dynamic block; and the dynamic block is raised to the residual launch's size
  static const bool attr_ok = [&] {
    hipFuncAttributes fa;
    const void* fn = reinterpret_cast<const void*>(dec_mfma_kernel<SUB, NW, R, SGN, ROPE, DQ>);
    return hipFuncGetAttributes(&fa, fn) == hipSuccess && fa.sharedSizeBytes == 0 &&
           hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_max) == hipSuccess;
  }();
  if (!attr_ok) return NSN_ERR_HIP;
  const int per = (((max_seq_len + n_splits - 1) / n_splits) + 63) & ~63;
  int* counters = static_cast<int*>(workspace);
  float* partial = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + counter_bytes);
  const dim3 grid(n_splits, g.n_kv_heads, batch);
  const int waves = res.k != nullptr ? NW + 1 : NW;  // + the residual wave
  dec_mfma_kernel<SUB, NW, R, SGN, ROPE, DQ><<<grid, waves * 64, smem, stream>>>(
      g, (const __half*)codebook, (const __half*)q, kv, vv, seq_lens, scale * 1.44269504088896340736f, n_splits,
      per, partial, counters, res, head_off, r_pass, out);
  return hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
}

// arrival counters sit at the head of the workspace: one per (sequence, query head), each on a 256-byte
// line of its own (atomic updates of one line are served one after the other, wherever in the line they
// fall); this kernel uses one per (sequence, kv head) of them, the tiled-layout kernel all
static size_t counter_bytes(const nsn_shape& s, int batch) {
  return (size_t)batch * s.n_q_heads * kCounterStrideInts * sizeof(int);
}
size_t decode_counter_bytes(const nsn_shape& s, int batch) { return counter_bytes(s, batch); }

int decode_mfma_splits(const nsn_shape& s, int batch, int max_seq_len, int requested) {
  const int cap = max(1, min(64, (max_seq_len + 255) / 256));
  if (requested > 0) return min(requested, 64);
  const int units = max(1, batch * s.n_kv_heads);
  // Half a chip's worth of units or more: splitting cannot even out a ragged batch any further (a split is a
  // workgroup with its own table and epilogue), the persistent instance can
  if (shape_is_tiled(s) && units >= 128) return kSplitsFlat;
  return max(1, min(cap, (256 + units - 1) / units));  // one 8-wave workgroup per compute unit
}

size_t decode_mfma_workspace_bytes(const nsn_shape& s, int batch, int n_splits) {
  // kSplitsFlat: two partials per run and query head of a kv head
  const size_t partials = n_splits == kSplitsFlat ? (size_t)kFlatRunsMax * 2 * (s.n_q_heads / s.n_kv_heads)
                                                  : (size_t)batch * s.n_q_heads * n_splits;
  return counter_bytes(s, batch) + partials * kPartialStrideM * sizeof(float);
}

int decode_mfma_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                       const nsn_cache& vc, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                       int n_splits, void* workspace, const nsn_residual* residual, float* out,
                       hipStream_t stream) {
  if (shape_is_tiled(s))
    return decode_tile_launch(s, codebook, q, kc, vc, seq_lens, batch, max_seq_len, scale, n_splits, workspace,
                              counter_bytes(s, batch), residual, out, stream);
  const Geometry g = make_geometry(s);
  ResidualView res = {nullptr, nullptr, nullptr, 0};
  if (residual)
    res = {static_cast<const __half*>(residual->k_fp16), static_cast<const __half*>(residual->v_fp16),
           residual->lens, residual->capacity};
  const CacheView kv = make_view(kc), vv = make_view(vc);
  const size_t cb = counter_bytes(s, batch);
  const int r_total = s.n_q_heads / s.n_kv_heads;
  // up to four query heads per kv head in one launch; five to eight as two launches on the same
  // stream (the second reads the cache again; partials and counters are reused in stream order)
  for (int head_off = 0; head_off < r_total; head_off += 4) {
    const int r = min(4, r_total - head_off);
#define NSN_ARGS \
  g, codebook, q, kv, vv, seq_lens, batch, max_seq_len, scale, n_splits, workspace, cb, res, head_off, r, out, stream
    // instance = (code format) x (heads of this launch: 1, 2, or 3-4) x (mean turned in the kernel) x (4-bit side information)
    auto with_r = [&](auto sub, auto sgn, auto rope, auto dq) {
      constexpr int kSub = decltype(sub)::value;
      constexpr bool kSgn = decltype(sgn)::value, kRope = decltype(rope)::value, kDq = decltype(dq)::value;
      if constexpr (kRope && kDq) {
        // Mean turned in the kernel AND 4-bit side information: with nine waves (168 registers each) these
        // instances spill 50-210 bytes per lane; with seven main waves the launch has at most eight, each
        // may use 256 registers, nothing spills, and they run 12-15 % faster in spite of the missing wave
        // (the instances with only one of the two options lose 2-8 % that way and keep eight).
        return r == 1   ? launch_one<kSub, 7, 1, kSgn, kRope, kDq>(NSN_ARGS)
               : r == 2 ? launch_one<kSub, 7, 2, kSgn, kRope, kDq>(NSN_ARGS)
                        : launch_one<kSub, 7, 4, kSgn, kRope, kDq>(NSN_ARGS);
      } else
        return r == 1   ? launch_one<kSub, 8, 1, kSgn, kRope, kDq>(NSN_ARGS)
               : r == 2 ? launch_one<kSub, 8, 2, kSgn, kRope, kDq>(NSN_ARGS)
                        : launch_one<kSub, 8, 4, kSgn, kRope, kDq>(NSN_ARGS);
    };
    auto with_format = [&](auto rope, auto dq) {
      if constexpr (!decltype(rope)::value) {
        // index-only codes without a rotary table run in the tiled-layout kernel (dispatched above), with
        // either width of side information; what is left here without the table is the sign + index format
        return g.sign ? with_r(std::integral_constant<int, 8>{}, std::true_type{}, rope, dq) : (int)NSN_ERR_UNSUPPORTED;
      }
      if (g.sign) return with_r(std::integral_constant<int, 8>{}, std::true_type{}, rope, dq);
      if (s.sub_dim == 4) return with_r(std::integral_constant<int, 4>{}, std::false_type{}, rope, dq);
      return with_r(std::integral_constant<int, 8>{}, std::false_type{}, rope, dq);
    };
    int rc;
    if (g.rope)
      rc = g.dq ? with_format(std::true_type{}, std::true_type{}) : with_format(std::true_type{}, std::false_type{});
    else
      rc = g.dq ? with_format(std::false_type{}, std::true_type{}) : with_format(std::false_type{}, std::false_type{});
#undef NSN_ARGS
    if (rc != NSN_OK) return rc;
  }
  return NSN_OK;
}

}  // namespace nsn
