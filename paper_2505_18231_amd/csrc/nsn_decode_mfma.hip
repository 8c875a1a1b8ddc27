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
//     fp32 accumulator is out_rot[head][channel] in the rotated domain.
// Partial results per (split, query head) go to the same fp32 layout the merge kernel reads.
#include <type_traits>

#include "nsn_host.h"

namespace nsn {

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kPartialStrideM = 2 * kHeadDim + 2;
constexpr float kLn2 = 0.69314718055994530942f;
constexpr float kLazyMaxLog2 = 5.0f;  // rescale only when a score beats the running max by 2^5
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

template <int SUB, int NW>
struct DecSmem {
  // codebook table: entry (code c, copy p) at c * 256 + p * (2 * SUB) bytes;
  // 32 copies of 8 B (SUB = 4) or 16 copies of 16 B (SUB = 8).  Reused by the epilogue.
  __attribute__((aligned(16))) unsigned char table[kTableBytes];
  float q_orig[4][kHeadDim];
  float q_had[4][kHeadDim];
  float accm[NW][4][kHeadDim];  // mean-vector term of every wave, original channel order
  float wave_m[NW][4], wave_l[NW][4];
};

template <int SUB, int NW>
__global__ __launch_bounds__(NW * 64) void dec_mfma_kernel(Geometry g, const __half* __restrict__ codebook,
                                                           const __half* __restrict__ q, CacheView kc,
                                                           CacheView vc, const int32_t* __restrict__ seq_lens,
                                                           float scale_log2e, int n_splits,
                                                           float* __restrict__ partial) {
  constexpr int J = kHeadDim / SUB;       // code bytes per token
  constexpr int KW = J / 4;               // code dwords per lane (K: one token; V: one sub-vector of J tokens)
  constexpr int LV = J;                   // lanes per value-side token part (one lane per sub-vector)
  constexpr int CBSZ_V = (SUB == 4) ? 3 : 2;
  constexpr int NT = NW * 64;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  auto& sm = *reinterpret_cast<DecSmem<SUB, NW>*>(smem_raw);

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int r = g.n_q_heads / g.n_kv_heads;  // <= 4
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int len = seq_lens[b];
  const int per = (((len + n_splits - 1) / n_splits) + 63) & ~63;
  const int t0 = split * per, t1 = min(len, t0 + per);
  float* P = partial + ((int64_t)(b * g.n_q_heads + h * r) * n_splits + split) * kPartialStrideM;
  if (t0 >= t1) {  // empty split
    for (int i = tid; i < r * 2 * kHeadDim; i += NT)
      P[(int64_t)(i / (2 * kHeadDim)) * n_splits * kPartialStrideM + (i % (2 * kHeadDim))] = 0.f;
    if (tid < r) {
      P[(int64_t)tid * n_splits * kPartialStrideM + 2 * kHeadDim] = -INFINITY;
      P[(int64_t)tid * n_splits * kPartialStrideM + 2 * kHeadDim + 1] = 0.f;
    }
    return;
  }

  // ---- prologue: replicated codebook table, rotated query ----------------------------------
  if constexpr (SUB == 4) {
    const uint2* cb2 = reinterpret_cast<const uint2*>(codebook);
    for (int i = tid; i < kCodes * 32; i += NT)
      *reinterpret_cast<uint2*>(sm.table + (i >> 5) * 256 + (i & 31) * 8) = cb2[i >> 5];
  } else {
    const uint4* cb4 = reinterpret_cast<const uint4*>(codebook);
    for (int i = tid; i < kCodes * 16; i += NT)
      *reinterpret_cast<uint4*>(sm.table + (i >> 4) * 256 + (i & 15) * 16) = cb4[i >> 4];
  }
  for (int i = tid; i < 4 * kHeadDim; i += NT) {
    const int hh = i >> 7, c = i & 127;
    const float v = hh < r ? __half2float(q[(int64_t)(b * g.n_q_heads + h * r + hh) * kHeadDim + c]) : 0.f;
    sm.q_orig[hh][c] = v;
    sm.q_had[hh][c] = v;
  }
  for (int s = 1; s < kHeadDim; s <<= 1) {  // d1: four 128-point Walsh-Hadamard transforms
    __syncthreads();
    for (int i = tid; i < 4 * 64; i += NT) {
      const int hh = i >> 6, k = i & 63;
      const int lo = ((k & ~(s - 1)) << 1) | (k & (s - 1));
      const float a0 = sm.q_had[hh][lo], a1 = sm.q_had[hh][lo + s];
      sm.q_had[hh][lo] = a0 + a1;
      sm.q_had[hh][lo + s] = a0 - a1;
    }
  }
  for (int i = tid; i < NW * 4 * kHeadDim; i += NT) (&sm.accm[0][0][0])[i] = 0.f;
  __syncthreads();

  // A operands of the score contraction: slot s = channels [4s, 4s+4); block (lane / 4) of
  // register pair p holds slot 16 p + block for head (lane % 4); fp16 hi and lo parts.
  const float qscale = (float)kInvSqrtD * scale_log2e;
  h4 QH[2], QL[2];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const float* src = &sm.q_had[lane & 3][4 * (16 * p + (lane >> 2))];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float x = src[k] * qscale;
      const _Float16 hi = (_Float16)x;
      QH[p][k] = hi;
      QL[p][k] = (_Float16)(x - (float)hi);
    }
  }
  const float qo0[4] = {sm.q_orig[0][2 * lane], sm.q_orig[1][2 * lane], sm.q_orig[2][2 * lane],
                        sm.q_orig[3][2 * lane]};
  const float qo1[4] = {sm.q_orig[0][2 * lane + 1], sm.q_orig[1][2 * lane + 1], sm.q_orig[2][2 * lane + 1],
                        sm.q_orig[3][2 * lane + 1]};

  const uint32_t laneoff = (SUB == 4) ? (lane & 31) * 8 : (lane & 15) * 16;
  const int64_t mean_base = (int64_t)(b * g.n_kv_heads + h) * g.n_groups_max;

  float m_run[4], l_run[4], beta[4], cf[4], qo[4];
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

  // flush the mean-vector term of the Shift group that just ended: accm = accm * cf + beta * o^v
  auto flush_group = [&](int grp) {
    const __half2 o2 = *reinterpret_cast<const __half2*>(vc.means + (mean_base + grp) * kHeadDim + 2 * lane);
    const float o0 = __low2float(o2), o1 = __high2float(o2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float bsum = xor_sum(beta[i], 64);
      float* dst = &sm.accm[wave][i][2 * lane];
      dst[0] = dst[0] * cf[i] + bsum * o0;
      dst[1] = dst[1] * cf[i] + bsum * o1;
      beta[i] = 0.f;
      cf[i] = 1.f;
    }
  };

  // ---- main loop: this wave's 64-token groups ---------------------------------------------
  const int n_grp = (t1 - t0 + 63) >> 6;
  for (int gi = wave; gi < n_grp; gi += NW) {
    const int tg = t0 + (gi << 6);  // first token of the group (multiple of 64)
    const int64_t kbase = unit_token_base(g, kc.block_table, b, h, tg);
    const int64_t vbase = unit_token_base(g, vc.block_table, b, h, tg);
    const int tin = token_in_unit(g, tg);
    const bool valid = (tg + lane) < t1;

    uint32_t kcode[KW], vcode[KW];
    {
      const uint4* kp = reinterpret_cast<const uint4*>(kc.codes + (kbase + tin + lane) * J);
      const uint4* vp = reinterpret_cast<const uint4*>(vc.codes + (vbase + tin) * J + (lane / LV) * (J * J) +
                                                       (lane % LV) * J);
#pragma unroll
      for (int w4 = 0; w4 < KW / 4; ++w4) {
        const uint4 kv4 = kp[w4], vv4 = vp[w4];
        kcode[4 * w4] = kv4.x, kcode[4 * w4 + 1] = kv4.y, kcode[4 * w4 + 2] = kv4.z, kcode[4 * w4 + 3] = kv4.w;
        vcode[4 * w4] = vv4.x, vcode[4 * w4 + 1] = vv4.y, vcode[4 * w4 + 2] = vv4.z, vcode[4 * w4 + 3] = vv4.w;
      }
    }
    const __half2 nk = kc.norms[kbase + tin + lane];
    const __half2 nv = vc.norms[vbase + tin + lane];
    const float a_k = valid ? __low2float(nk) : 0.f, b_k = valid ? __high2float(nk) : 0.f;
    const float a_v = valid ? __low2float(nv) : 0.f, b_v = valid ? __high2float(nv) : 0.f;

    // Shift group bookkeeping (wave-uniform): q . o^k of the new group, mean term of the old one
    const int grp = group_of(g, tg);
    if (grp != cur_group) {
      if (cur_group >= 0) flush_group(cur_group);
      const __half2 o2 = *reinterpret_cast<const __half2*>(kc.means + (mean_base + grp) * kHeadDim + 2 * lane);
      const float o0 = __low2float(o2), o1 = __high2float(o2);
#pragma unroll
      for (int i = 0; i < 4; ++i) qo[i] = xor_sum(qo0[i] * o0 + qo1[i] * o1, 64) * scale_log2e;
      cur_group = grp;
    }

    // d2/d3: HT(q) . C[codes] for four heads, fp32 accumulate over the sub-vectors
    f4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (SUB == 4) {
      static_for<32>([&](auto ic) {
        constexpr int s = decltype(ic)::value;
        const uint32_t addr = perm_b32(kcode[s / 4], laneoff, 0x0c0c0400u + ((s % 4) << 8));
        const uint2 cw = *reinterpret_cast<const uint2*>(sm.table + addr);
        const h4 bop = as_h4(cw.x, cw.y);
        d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(QH[s / 16], bop, d0, 4, s % 16, 0);
        d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(QL[s / 16], bop, d1, 4, s % 16, 0);
      });
    } else {
      static_for<16>([&](auto ic) {
        constexpr int s = decltype(ic)::value;
        const uint32_t addr = perm_b32(kcode[s / 4], laneoff, 0x0c0c0400u + ((s % 4) << 8));
        const uint4 cw = *reinterpret_cast<const uint4*>(sm.table + addr);
        const h4 b0 = as_h4(cw.x, cw.y), b1 = as_h4(cw.z, cw.w);
        d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(QH[(2 * s) / 16], b0, d0, 4, (2 * s) % 16, 0);
        d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(QL[(2 * s) / 16], b0, d1, 4, (2 * s) % 16, 0);
        d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(QH[(2 * s + 1) / 16], b1, d0, 4, (2 * s + 1) % 16, 0);
        d1 = __builtin_amdgcn_mfma_f32_4x4x4f16(QL[(2 * s + 1) / 16], b1, d1, 4, (2 * s + 1) % 16, 0);
      });
    }

    // d3/d4: scores in log2 units, lazy running max, weights
    float s[4], w[4];
    bool need = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s[i] = valid ? fmaf(a_k, d0[i] + d1[i], b_k * qo[i]) : -INFINITY;
      need = need || (s[i] - m_run[i] > kLazyMaxLog2);
    }
    if (__any(need)) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float m_new = fmaxf(m_run[i], wave_max(s[i]));
        const float corr = (m_run[i] == -INFINITY) ? 0.f : fast_exp2(m_run[i] - m_new);
        l_run[i] *= corr;
        beta[i] *= corr;
        cf[i] *= corr;
#pragma unroll
        for (int c = 0; c < SUB; ++c) acc[c][i] *= corr;
        m_run[i] = m_new;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float p = fast_exp2(s[i] - m_run[i]);  // 0 for masked lanes
      l_run[i] += p;
      beta[i] = fmaf(p, b_v, beta[i]);
      w[i] = p * a_v;
    }
    quad_transpose(w, lane);  // lane i of a quad: head i, the quad's four tokens
    h4 wop;
#pragma unroll
    for (int k = 0; k < 4; ++k) wop[k] = (_Float16)w[k];

    // d5: out_rot[head][channel] += sum over tokens of weight * codeword channel
    static_for<KW>([&](auto ic) {
      constexpr int a = decltype(ic)::value;
      const uint32_t vw = vcode[a];
      if constexpr (SUB == 4) {
        uint2 cw[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
          cw[k] = *reinterpret_cast<const uint2*>(sm.table + perm_b32(vw, laneoff, 0x0c0c0400u + (k << 8)));
        const h4 b0 = as_h4(perm_b32(cw[1].x, cw[0].x, 0x05040100u), perm_b32(cw[3].x, cw[2].x, 0x05040100u));
        const h4 b1 = as_h4(perm_b32(cw[1].x, cw[0].x, 0x07060302u), perm_b32(cw[3].x, cw[2].x, 0x07060302u));
        const h4 b2 = as_h4(perm_b32(cw[1].y, cw[0].y, 0x05040100u), perm_b32(cw[3].y, cw[2].y, 0x05040100u));
        const h4 b3 = as_h4(perm_b32(cw[1].y, cw[0].y, 0x07060302u), perm_b32(cw[3].y, cw[2].y, 0x07060302u));
        acc[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b0, acc[0], CBSZ_V, a, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b1, acc[1], CBSZ_V, a, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b2, acc[2], CBSZ_V, a, 0);
        acc[3] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, b3, acc[3], CBSZ_V, a, 0);
      } else {
        uint4 cw[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
          cw[k] = *reinterpret_cast<const uint4*>(sm.table + perm_b32(vw, laneoff, 0x0c0c0400u + (k << 8)));
        const uint32_t c0[4] = {cw[0].x, cw[0].y, cw[0].z, cw[0].w};
        const uint32_t c1[4] = {cw[1].x, cw[1].y, cw[1].z, cw[1].w};
        const uint32_t c2[4] = {cw[2].x, cw[2].y, cw[2].z, cw[2].w};
        const uint32_t c3[4] = {cw[3].x, cw[3].y, cw[3].z, cw[3].w};
#pragma unroll
        for (int mth = 0; mth < 4; ++mth) {
          const h4 be = as_h4(perm_b32(c1[mth], c0[mth], 0x05040100u), perm_b32(c3[mth], c2[mth], 0x05040100u));
          const h4 bo = as_h4(perm_b32(c1[mth], c0[mth], 0x07060302u), perm_b32(c3[mth], c2[mth], 0x07060302u));
          acc[2 * mth] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, be, acc[2 * mth], CBSZ_V, a, 0);
          acc[2 * mth + 1] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, bo, acc[2 * mth + 1], CBSZ_V, a, 0);
        }
      }
    });
  }
  if (cur_group >= 0) flush_group(cur_group);

  // ---- epilogue: wave results -> LDS (reusing the table), merge the waves, write partials ---
#pragma unroll
  for (int i = 0; i < 4; ++i) l_run[i] = xor_sum(l_run[i], 64);
#pragma unroll
  for (int c = 0; c < SUB; ++c)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = acc[c][i];
      for (int msk = LV; msk < 64; msk <<= 1) v += __shfl_xor(v, msk, 64);
      acc[c][i] = v;
    }
  __syncthreads();  // every wave is done gathering from the table
  float* racc = reinterpret_cast<float*>(sm.table);  // [NW][4][128]
  if (lane < LV) {
#pragma unroll
    for (int c = 0; c < SUB; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) racc[(wave * 4 + i) * kHeadDim + lane * SUB + c] = acc[c][i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (lane == i) {
      sm.wave_m[wave][i] = m_run[i];
      sm.wave_l[wave][i] = l_run[i];
    }
  __syncthreads();
  for (int i = tid; i < r * kHeadDim; i += NT) {
    const int hh = i >> 7, c = i & 127;
    float M = -INFINITY;
    for (int wv = 0; wv < NW; ++wv) M = fmaxf(M, sm.wave_m[wv][hh]);
    float L = 0.f, orot = 0.f, omean = 0.f;
    for (int wv = 0; wv < NW; ++wv) {
      const float mw = sm.wave_m[wv][hh];
      const float e = (mw == -INFINITY) ? 0.f : fast_exp2(mw - M);
      L = fmaf(e, sm.wave_l[wv][hh], L);
      orot = fmaf(e, racc[(wv * 4 + hh) * kHeadDim + c], orot);
      omean = fmaf(e, sm.accm[wv][hh][c], omean);
    }
    float* Ph = P + (int64_t)hh * n_splits * kPartialStrideM;
    Ph[c] = orot;
    Ph[kHeadDim + c] = omean;
    if (c == 0) {
      Ph[2 * kHeadDim] = M * kLn2;
      Ph[2 * kHeadDim + 1] = L;
    }
  }
}

// ---------------------------------------------------------------------------------------
template <int SUB, int NW>
static int launch_one(const Geometry& g, const void* codebook, const void* q, const CacheView& kv,
                      const CacheView& vv, const int32_t* seq_lens, int batch, float scale, int n_splits,
                      float* partial, hipStream_t stream) {
  const size_t smem = sizeof(DecSmem<SUB, NW>);
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(dec_mfma_kernel<SUB, NW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return NSN_ERR_HIP;
    attr_done = true;
  }
  const dim3 grid(n_splits, g.n_kv_heads, batch);
  dec_mfma_kernel<SUB, NW><<<grid, NW * 64, smem, stream>>>(g, (const __half*)codebook, (const __half*)q, kv, vv,
                                                            seq_lens, scale * 1.44269504088896340736f, n_splits,
                                                            partial);
  return NSN_OK;
}

int decode_mfma_splits(const nsn_shape& s, int batch, int max_seq_len, int requested) {
  const int cap = max(1, min(64, (max_seq_len + 255) / 256));
  if (requested > 0) return min(requested, 64);
  const int units = max(1, batch * s.n_kv_heads);
  return max(1, min(cap, (512 + units - 1) / units));  // about two workgroups per compute unit
}

int decode_mfma_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                       const nsn_cache& vc, const int32_t* seq_lens, int batch, float scale, int n_splits,
                       float* partial, hipStream_t stream) {
  const Geometry g = make_geometry(s);
  const CacheView kv = make_view(kc), vv = make_view(vc);
  return s.sub_dim == 4 ? launch_one<4, 4>(g, codebook, q, kv, vv, seq_lens, batch, scale, n_splits, partial, stream)
                        : launch_one<8, 4>(g, codebook, q, kv, vv, seq_lens, batch, scale, n_splits, partial, stream);
}

}  // namespace nsn
