// KV encoder kernels: Normalize - Shift - Normalize (Sec. 3.2), Hadamard rotation (Sec. 2),
// nearest-codeword search (Eq. 1), scale adjustment (Sec. 3.3).
//
// Three launches per call:
//   enc_stats_kernel  per token: b = fp16(||x|| / sqrt(d)); per chunk: fp64 partial sums of x / b
//   enc_means_kernel  per group: o = fp16(sum of partials / count)           (skipped in append mode)
//   enc_quant_kernel  per token: (x / b - o) -> s2 -> rotate -> codes, a = fp16(b * s2 * alpha)
// Double quantization (Sec. 3.5, side_bits = 4): enc_stats_kernel leaves fp16(s1) in the workspace,
// enc_brtn_kernel turns every 64-token block of them into 4-bit codes, enc_means_kernel stores the
// means as 4-bit codes per 32 channels, and enc_quant_kernel shifts by the dequantised mean and
// stores a' = fp16(s2 * alpha).
// Normalisation, rotation and the dot products that feed fp16 roundings run in fp64 (same rate
// as fp32 on this chip's vector units); only the 256-way distance scan runs in fp32.
#include "nsn_host.h"
#include <cstdlib>
#include <type_traits>

#include "nsn_vq_mfma.h"

namespace nsn {

// f(integral_constant<int, m>) for m = 1, 2, 4, ... < N
template <int N, int M = 1, typename F>
__device__ __forceinline__ void static_for_pow2(F&& f) {
  if constexpr (M < N) {
    f(std::integral_constant<int, M>{});
    static_for_pow2<N, M * 2>(f);
  }
}

// ---------------------------------------------------------------------------------------
// Stage A: first Normalize scale per token, partial channel sums of the normalised tokens.
// grid (chunk, kv_head * 2 + tensor, sequence), block 256 = 4 waves; a wave takes four tokens at a
// time (sixteen lanes per token, a lane owns eight consecutive channels: one 16-byte load).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void enc_stats_kernel(Geometry g, const __half* __restrict__ k_in,
                                                        const __half* __restrict__ v_in, int max_new,
                                                        int max_len, const int32_t* __restrict__ seq_start,
                                                        const int32_t* __restrict__ n_new, CacheView kc,
                                                        CacheView vc, double* __restrict__ partial,
                                                        int chunk_tokens, int n_chunks, __half* __restrict__ ws_b) {
  const int chunk = blockIdx.x, h = blockIdx.y >> 1, tensor = blockIdx.y & 1, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane >> 4, col = lane & 15;  // token of the wave's four, channels [8 col, 8 col + 8)
  const CacheView& cv = tensor ? vc : kc;
  const __half* in = (tensor ? v_in : k_in) + ((int64_t)(b * g.n_kv_heads + h) * max_new) * kHeadDim;
  __half* wsb = ws_b + ((int64_t)(b * g.n_kv_heads + h) * 2 + tensor) * max_new;  // side_bits = 4 only
  const int start = seq_start[b];
  const int count = min(min(n_new[b], max_new), max_len - start);  // tokens that have a place in the cache
  const int t_end = min((chunk + 1) * chunk_tokens, count);

  double acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0;
  // four steps of loads in flight; a token past the end is read from the last valid row (the chunk has at
  // least one: t_end > chunk start, or the loop below does not run) and its weight is set to zero
  auto fetch = [&](int t) -> uint4 {
    return *reinterpret_cast<const uint4*>(in + (int64_t)min(t, max(t_end - 1, 0)) * kHeadDim + 8 * col);
  };
  // where fp16(s1) of token t goes: one address that is linear in t, except for paged caches
  const bool linear = g.dq || !g.paged;  // uniform
  __half* const b_out = g.dq ? wsb
                             : reinterpret_cast<__half*>(cv.norms) +
                                   2 * ((int64_t)(b * g.n_kv_heads + h) * g.page_tokens + start) + 1;
  const int b_stride = g.dq ? 1 : 2;
  auto step = [&](const uint4 raw, int t) {
    const __half* xh = reinterpret_cast<const __half*>(&raw);
    double x[8], ss = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      x[i] = (double)__half2float(xh[i]);
      ss = fma(x[i], x[i], ss);
    }
    ss = xor_sum_w<16>(ss);
    // s1 = sqrt(ss / d) and 1 / fp16(s1) by the hardware estimates and Newton steps (ss is a sum of squares
    // of fp16 values: zero or far inside the fp64 range, so no scaling is needed).  Both are within an fp64
    // unit or two of the correctly rounded values; what is stored is rounded to fp16.
    const double sd = ss * (1.0 / kHeadDim);
    double s1 = 0.0;
    if (sd != 0.0) {
      const double y = __builtin_amdgcn_rsq(sd);
      double gq = sd * y, hq = 0.5 * y;
      const double r0 = fma(-hq, gq, 0.5);
      gq = fma(gq, r0, gq), hq = fma(hq, r0, hq);
      s1 = fma(fma(-gq, gq, sd), hq, gq);
    }
    const __half b16 = f64_to_f16(s1);
    const double bb = (double)__half2float(b16);
    double rb = 0.0;  // (tokens past the end add nothing)
    if (bb != 0.0 && t < t_end) {
      rb = __builtin_amdgcn_rcp(bb);
      rb = fma(fma(-bb, rb, 1.0), rb, rb);
      rb = fma(fma(-bb, rb, 1.0), rb, rb);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = fma(x[i], rb, acc[i]);
    if (col == 0 && t < t_end) {
      if (linear) {
        b_out[(int64_t)t * b_stride] = b16;
      } else {
        const int pos = start + t;
        const int64_t base = unit_token_base(g, cv.block_table, b, h, pos);
        reinterpret_cast<__half*>(cv.norms)[2 * (base + token_in_unit(g, pos)) + 1] = b16;
      }
    }
  };
  // the four buffers are refilled in place, four steps to a round (no register moves between steps)
  const int tw = chunk * chunk_tokens + 4 * wave;  // the wave's first token of a step (uniform)
  uint4 buf[4] = {fetch(tw + row), fetch(tw + row + 16), fetch(tw + row + 32), fetch(tw + row + 48)};
  for (int t0 = tw; t0 < t_end; t0 += 64) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (t0 + 16 * u < t_end) {  // wave-uniform
        const uint4 raw = buf[u];
        buf[u] = fetch(t0 + 16 * u + row + 64);
        step(raw, t0 + 16 * u + row);
      }
    }
  }
  // the wave's four token rows, then the four waves
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    acc[i] += xor_lane<16>(acc[i]);
    acc[i] += xor_lane<32>(acc[i]);
  }
  __shared__ double red[4][kHeadDim];
  if (row == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) red[wave][8 * col + i] = acc[i];
  }
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    const int c = threadIdx.x;
    const double s = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
    partial[((((int64_t)(b * g.n_kv_heads + h) * 2 + tensor) * n_chunks) + chunk) * kHeadDim + c] = s;
  }
}

// 4-bit round-to-nearest levels of one group (Sec. 3.5): minimum and step in fp16, the code of x taken
// against the rounded minimum and step
__device__ inline int rtn4_code(double x, double mn, double st) {
  if (st == 0.0) return 0;
  const double lvl = floor((x - mn) / st + 0.5);
  return (int)fmin(fmax(lvl, 0.0), 15.0);
}

// ---------------------------------------------------------------------------------------
// Stage A1 (side_bits = 4): 4-bit codes of fp16(s1) per 64-token block.  grid (64-token block of the
// call, kv_head * 2 + tensor, sequence), block 64: a lane owns one token.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void enc_brtn_kernel(Geometry g, int max_new, int max_len,
                                                      const int32_t* __restrict__ seq_start,
                                                      const int32_t* __restrict__ n_new, CacheView kc, CacheView vc,
                                                      const __half* __restrict__ ws_b) {
  const int h = blockIdx.y >> 1, tensor = blockIdx.y & 1, b = blockIdx.z;
  const int lane = threadIdx.x;
  const CacheView& cv = tensor ? vc : kc;
  const int start = seq_start[b];
  const int count = min(n_new[b], max_new);
  const int t = blockIdx.x * 64 + lane, pos = start + t;
  const bool valid = t < count && pos < max_len;
  if (blockIdx.x * 64 >= count || start + blockIdx.x * 64 >= max_len) return;  // uniform: lane 0 is valid below
  const float x = valid ? __half2float(ws_b[((int64_t)(b * g.n_kv_heads + h) * 2 + tensor) * max_new + t]) : 0.f;
  float lo = valid ? x : INFINITY, hi = valid ? x : -INFINITY;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    lo = fminf(lo, __shfl_xor(lo, m, 64));
    hi = fmaxf(hi, __shfl_xor(hi, m, 64));
  }
  const __half mn16 = f64_to_f16((double)lo);  // exact: the minimum is one of the fp16 inputs
  const __half st16 = f64_to_f16(((double)hi - (double)lo) / 15.0);
  const int code = valid ? rtn4_code((double)x, (double)__half2float(mn16), (double)__half2float(st16)) : 0;
  const int other = __shfl_xor(code, 1, 64);
  const int pos0 = start + blockIdx.x * 64;  // the block's first token (the record is chosen by it)
  unsigned char* rec = dq_norm_rec(cv, unit_token_base(g, cv.block_table, b, h, pos0), token_in_unit(g, pos0));
  if ((lane & 1) == 0 && valid) rec[kDqNormCodes + (lane >> 1)] = (unsigned char)(code | (other << 4));
  if (lane == 0) *reinterpret_cast<__half2*>(rec + kDqNormPar) = __halves2half2(mn16, st16);
}

// ---------------------------------------------------------------------------------------
// Stage A2: Shift vector of every new group.  grid (group-in-call, kv_head * 2 + tensor, sequence),
// block 128 (one thread per channel); partial sums are added in chunk order.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void enc_means_kernel(Geometry g, int max_new, int max_len,
                                                        const int32_t* __restrict__ seq_start,
                                                        const int32_t* __restrict__ n_new, CacheView kc,
                                                        CacheView vc, const double* __restrict__ partial,
                                                        int chunk_tokens, int n_chunks) {
  const int gl = blockIdx.x, h = blockIdx.y >> 1, tensor = blockIdx.y & 1, b = blockIdx.z;
  const int c = threadIdx.x;
  const CacheView& cv = tensor ? vc : kc;
  const int start = seq_start[b];
  const int count = min(min(n_new[b], max_new), max_len - start);
  int first_chunk, last_chunk, tokens, g_abs;
  if (g.group_size > 0) {  // chunk_tokens == group_size
    first_chunk = gl;
    last_chunk = gl + 1;
    tokens = min(g.group_size, count - gl * g.group_size);
    g_abs = start / g.group_size + gl;
  } else {
    first_chunk = 0;
    last_chunk = (count + chunk_tokens - 1) / chunk_tokens;
    tokens = count;
    g_abs = 0;
  }
  if (tokens <= 0 || g_abs >= g.n_groups_max) return;
  const double* p = partial + (((int64_t)(b * g.n_kv_heads + h) * 2 + tensor) * n_chunks) * kHeadDim + c;
  double s = 0.0;
  // added in chunk order, loaded eight at a time (one load per addition would be one memory round
  // trip per chunk: 512 of them for a 131072-token sequence)
  for (int k0 = first_chunk; k0 < last_chunk; k0 += 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (k0 + u < last_chunk) ? p[(int64_t)(k0 + u) * kHeadDim] : 0.0;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (k0 + u < last_chunk) s += v[u];
  }
  const double mean = s / (double)tokens;
  const int64_t mean_index = (int64_t)(b * g.n_kv_heads + h) * g.n_groups_max + g_abs;
  if (!g.dq) {
    cv.means[mean_index * kHeadDim + c] = f64_to_f16(mean);
    return;
  }
  // side_bits = 4: 16 levels per 32 channels (half a wave)
  double lo = mean, hi = mean;
#pragma unroll
  for (int m = 1; m < 32; m <<= 1) {
    lo = fmin(lo, __shfl_xor(lo, m, 64));
    hi = fmax(hi, __shfl_xor(hi, m, 64));
  }
  const __half mn16 = f64_to_f16(lo), st16 = f64_to_f16((hi - lo) / 15.0);
  const int code = rtn4_code(mean, (double)__half2float(mn16), (double)__half2float(st16));
  const int other = __shfl_xor(code, 1, 64);
  unsigned char* rec = dq_mean_rec(cv, mean_index);
  if ((c & 1) == 0) rec[c >> 1] = (unsigned char)(code | (other << 4));
  if ((c & 31) == 0) *reinterpret_cast<__half2*>(rec + kDqMeanPar + 4 * (c >> 5)) = __halves2half2(mn16, st16);
}

// ---------------------------------------------------------------------------------------
// Stage B: shift, second Normalize, rotation, search, scale adjustment, stores.
// grid (64- or 16-token chunk, kv_head * 2 + tensor, sequence), block 256.  A lane owns one
// sub-vector (SUB channels) of one token; a wave covers 64 / J tokens at a time.
// ---------------------------------------------------------------------------------------
// MFMA:  distance contraction on the matrix cores (else the fp32 vector-ALU scan)
// FUSED: append mode - the first-Normalize scale is computed here instead of by the stats kernel
// The register budget is pinned to the main path's needs (4 waves per SIMD at sub-vector length 4,
// 3 at length 8): without it the rarely taken re-listing path is scheduled for maximum
// instruction-level parallelism and doubles the register count of the whole kernel.
// SIGN:  the paper's 2-bit format (Sec. 3.4): the search runs on the absolute values against a
//        codebook of magnitudes; byte row jj holds the index, byte row 16 + jj the eight sign bits
// ROPE:  the K rows are keys before the rotary embedding (Sec. 3.2 "NSN applied to key and value"):
//        v_nsn is turned by the token's position between the second Normalize and the Hadamard rotation
template <int SUB, bool MFMA, bool FUSED, bool SIGN = false, bool ROPE = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(SUB == 4 ? 4 : 3))) void enc_quant_kernel(Geometry g, const __half* __restrict__ codebook,
                                                        const __half* __restrict__ k_in,
                                                        const __half* __restrict__ v_in, int max_new,
                                                        int max_len, const int32_t* __restrict__ seq_start,
                                                        const int32_t* __restrict__ n_new, CacheView kc,
                                                        CacheView vc, int wave_tokens,
                                                        const __half* __restrict__ ws_b) {
  // wave_tokens: tokens per wave (16, or 4 when the call is too small to fill the chip with 64-token blocks)
  constexpr int J = kHeadDim / SUB;  // lanes per token
  constexpr int TPW = 64 / J;        // tokens per wave step
  constexpr int JB = SIGN ? 2 * J : J;  // code bytes per token
  static_assert(!SIGN || SUB == 8, "the sign + index format is defined on 8-dim sub-vectors");
  __shared__ VqTables<SUB> T;
  const int h = blockIdx.y >> 1, tensor = blockIdx.y & 1, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jj = lane % J, tk = lane / J;
  const CacheView& cv = tensor ? vc : kc;
  const __half* in = (tensor ? v_in : k_in) + ((int64_t)(b * g.n_kv_heads + h) * max_new) * kHeadDim;
  const int start = seq_start[b];
  const int count = min(n_new[b], max_new);
  const int t_begin = blockIdx.x * (4 * wave_tokens) + wave * wave_tokens;

  // One token's inputs as this lane needs them (vector loads of SUB fp16 values); the first
  // token's loads are issued before the codebook tables are built, later ones one step ahead.
  typedef typename std::conditional<SUB == 4, uint2, uint4>::type vec_t;
  struct Tok {
    bool valid;
    int64_t base;
    int tin, pos;
    vec_t xraw, oraw;
    __half b16;
    uint32_t oq;  // side_bits = 4: the SUB 4-bit codes of this lane's channels of the mean
    __half2 op;   //                (min, step) of their 32-channel group
  };
  auto fetch = [&](int it) {
    Tok k;
    const int t = t_begin + it * TPW + tk;
    const int pos = start + t;
    k.valid = (t < count) && (pos < max_len);
    k.pos = pos;
    k.base = 0;
    k.tin = 0;
    k.xraw = vec_t{};
    k.oraw = vec_t{};
    k.b16 = __float2half(0.f);
    k.oq = 0u;
    k.op = __half2{};
    if (k.valid) {
      k.base = unit_token_base(g, cv.block_table, b, h, pos);
      k.tin = token_in_unit(g, pos);
      k.xraw = *reinterpret_cast<const vec_t*>(in + (int64_t)t * kHeadDim + jj * SUB);
      const int64_t mean_index =
          (int64_t)(b * g.n_kv_heads + h) * g.n_groups_max + min(group_of(g, pos), g.n_groups_max - 1);
      if (g.dq) {
        const unsigned char* rec = dq_mean_rec(cv, mean_index);
        if constexpr (SUB == 4)
          k.oq = *reinterpret_cast<const uint16_t*>(rec + jj * 2);
        else
          k.oq = *reinterpret_cast<const uint32_t*>(rec + jj * 4);
        k.op = *reinterpret_cast<const __half2*>(rec + kDqMeanPar + 4 * ((jj * SUB) >> 5));
        if constexpr (!FUSED) k.b16 = ws_b[((int64_t)(b * g.n_kv_heads + h) * 2 + tensor) * max_new + t];
      } else {
        k.oraw = *reinterpret_cast<const vec_t*>(cv.means + mean_index * kHeadDim + jj * SUB);
        if constexpr (!FUSED) k.b16 = reinterpret_cast<const __half*>(cv.norms)[2 * (k.base + k.tin) + 1];
      }
    }
    return k;
  };
  Tok nxt = fetch(0);

  vq_tables_fill<SUB>(T, [&](int c, int i) { return (double)__half2float(codebook[c * SUB + i]); });
  MfmaCodebook<SUB> MC;
  if constexpr (MFMA) mfma_codebook_load<SUB>(MC, T, lane);
  if (blockIdx.x * (4 * wave_tokens) >= count) return;

  const int n_it = wave_tokens / TPW;
  for (int it = 0; it < n_it; ++it) {
    if (t_begin + it * TPW >= count) break;  // wave-uniform: nothing left for this wave
    const Tok cur = nxt;
    if (it + 1 < n_it && t_begin + (it + 1) * TPW < count) nxt = fetch(it + 1);
    const bool valid = cur.valid;
    const int64_t base = cur.base;
    const int tin = cur.tin;
    const vec_t xraw = cur.xraw, oraw = cur.oraw;
    __half b16f = cur.b16;
    double xs[SUB], os[SUB];
    {
      const __half* xh = reinterpret_cast<const __half*>(&xraw);
      const __half* oh = reinterpret_cast<const __half*>(&oraw);
#pragma unroll
      for (int i = 0; i < SUB; ++i) {
        xs[i] = (double)__half2float(xh[i]);
        os[i] = (double)__half2float(oh[i]);
      }
      if (g.dq) {  // dequantised mean: min + step * code
        const double mn = (double)__low2float(cur.op), st = (double)__high2float(cur.op);
#pragma unroll
        for (int i = 0; i < SUB; ++i) os[i] = mn + st * (double)((cur.oq >> (4 * i)) & 15u);
      }
    }
    if constexpr (FUSED) {  // first Normalize here: b = fp16(||x|| / sqrt(d)), stored with the token
      double ssx = 0.0;
#pragma unroll
      for (int i = 0; i < SUB; ++i) ssx += xs[i] * xs[i];
      ssx = xor_sum_w<J>(ssx);
      b16f = f64_to_f16(sqrt(ssx) / kSqrtD);
      if (valid && jj == 0 && !g.dq) reinterpret_cast<__half*>(cv.norms)[2 * (base + tin) + 1] = b16f;
    }
    const double bb = (double)__half2float(b16f);
    // one division per token instead of one per channel: x * (1 / b) is within one fp64 unit of x / b, eight
    // decimal orders below anything the fp16 results and the code decisions can see
    const double rb = bb != 0.0 ? 1.0 / bb : 0.0;
    double v[SUB];
#pragma unroll
    for (int i = 0; i < SUB; ++i) v[i] = valid ? xs[i] * rb - os[i] : 0.0;
    // second Normalize
    double ss = 0.0;
#pragma unroll
    for (int i = 0; i < SUB; ++i) ss += v[i] * v[i];
    ss = xor_sum_w<J>(ss);
    const double s2 = sqrt(ss) * kInvSqrtD;  // (feeds the stored scale a, compared to one fp16 unit)
    const double r2 = (s2 != 0.0) ? 1.0 / s2 : 0.0;
#pragma unroll
    for (int i = 0; i < SUB; ++i) v[i] *= r2;
    if constexpr (ROPE) {
      if (tensor == 0) {  // keys only; the partner channel c ^ 64 lives in lane jj ^ (J / 2)
        // cos / sin of position * inv_freq[pair] from the fp64 table: block part and in-block part
        // combined by the addition theorems
        const int pc = min(max(cur.pos, 0), max_len - 1);  // lanes without a token hold zeros; keep them in bounds
        const int pair0 = (jj % (J / 2)) * SUB;
        const double2* blk = reinterpret_cast<const double2*>(g.rope + kRopeBlkOff +
                                                              (int64_t)(pc >> 6) * kRopeBlkStride + kRopeBlk64) + pair0;
        const double2* inb = reinterpret_cast<const double2*>(g.rope + kRopeInOff) + (pc & 63) * 64 + pair0;
        const bool upper = jj >= J / 2;
#pragma unroll
        for (int i = 0; i < SUB; ++i) {
          const double other = xor_lane<J / 2>(v[i]);
          const double2 c0 = blk[i], cj = inb[i];
          const double c = c0.x * cj.x - c0.y * cj.y, sn = c0.y * cj.x + c0.x * cj.y;
          v[i] = upper ? v[i] * c + other * sn : v[i] * c - other * sn;
        }
      }
    }
    // Walsh-Hadamard butterflies: channel bits 0..log2(SUB)-1 in registers, the rest across lanes
#pragma unroll
    for (int s = 1; s < SUB; s <<= 1) {
#pragma unroll
      for (int i = 0; i < SUB; ++i) {
        if ((i & s) == 0) {
          const double a0 = v[i], a1 = v[i | s];
          v[i] = a0 + a1;
          v[i | s] = a0 - a1;
        }
      }
    }
    static_for_pow2<J>([&](auto mc) {
      constexpr int m = decltype(mc)::value;
      const bool upper = (jj & m) != 0;
#pragma unroll
      for (int i = 0; i < SUB; ++i) {
        const double other = xor_lane<m>(v[i]);
        v[i] = upper ? other - v[i] : v[i] + other;
      }
    });
    double y[SUB];
#pragma unroll
    for (int i = 0; i < SUB; ++i) y[i] = v[i] * kInvSqrtD;

    // sign + index format: the nearest signed codeword has the signs of y and the magnitude
    // codeword nearest to |y| (the magnitudes are non-negative), and y . y_Q = |y| . C[code]
    double ys[SUB];
    uint32_t sign_byte = 0u;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      ys[i] = SIGN ? fabs(y[i]) : y[i];
      if (SIGN && y[i] < 0.0) sign_byte |= 1u << i;
    }
    int code;
    if constexpr (MFMA)
      code = vq_search_mfma<SUB>(T, MC, ys, lane);
    else
      code = vq_search<SUB>(T, ys);

    // scale adjustment: alpha = ||y||^2 / (y . y_Q)
    double dot = 0.0, nrm2 = 0.0;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      dot += ys[i] * T.cx[code][i];
      nrm2 += y[i] * y[i];
    }
    dot = xor_sum_w<J>(dot);
    nrm2 = xor_sum_w<J>(nrm2);
    const double alpha = (dot > 1e-12 * kHeadDim) ? nrm2 / dot : 1.0;
    if (valid) {
      const int64_t off = code_offset(g.tiled, tensor != 0, JB, tin, jj);
      cv.codes[base * JB + off] = (uint8_t)code;
      if constexpr (SIGN) {
        const int64_t soff = code_offset(g.tiled, tensor != 0, JB, tin, J + jj);
        cv.codes[base * JB + soff] = (uint8_t)sign_byte;
      }
      if (jj == 0) {
        if (g.dq)  // a' = fp16(s2 alpha); s1 is stored separately as a 4-bit code
          reinterpret_cast<__half*>(dq_norm_rec(cv, base, tin))[tin & 63] = f64_to_f16(s2 * alpha);
        else
          reinterpret_cast<__half*>(cv.norms)[2 * (base + tin)] = f64_to_f16(bb * s2 * alpha);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static int encode_chunk_tokens(const nsn_shape& s) { return s.group_size > 0 ? s.group_size : 256; }

static size_t encode_partial_bytes(const nsn_shape& s, int batch, int64_t max_new) {
  const int ct = encode_chunk_tokens(s);
  const int64_t n_chunks = (max_new + ct - 1) / ct;
  return (size_t)batch * s.n_kv_heads * 2 * n_chunks * kHeadDim * sizeof(double);
}

size_t encode_workspace_bytes(const nsn_shape& s, int batch, int64_t max_new) {
  // side_bits = 4: fp16(s1) of every new token passes through the workspace
  const size_t b_bytes = s.side_bits == 4 ? (((size_t)batch * s.n_kv_heads * 2 * max_new * sizeof(__half)) + 255) & ~(size_t)255 : 0;
  return encode_partial_bytes(s, batch, max_new) + b_bytes;
}

int encode_launch(const nsn_shape& s, const void* codebook, const void* k_in, const void* v_in, int max_new,
                  const int32_t* seq_start, const int32_t* n_new, int batch, int freeze_means,
                  const nsn_cache& kc, const nsn_cache& vc, void* workspace, hipStream_t stream) {
  const Geometry g = make_geometry(s);
  const CacheView kv = make_view(kc), vv = make_view(vc);
  const int ct = encode_chunk_tokens(s);
  const int n_chunks = (max_new + ct - 1) / ct;
  double* partial = static_cast<double*>(workspace);
  __half* ws_b = reinterpret_cast<__half*>(static_cast<unsigned char*>(workspace) + encode_partial_bytes(s, batch, max_new));
  const bool use_mfma = selected_variant(NSN_OP_ENCODE) != NSN_VARIANT_ALT;  // the alternative is the vector-ALU scan
  if (!freeze_means || g.dq) {  // side_bits = 4: the s1 codes of a block need all its tokens first
    const dim3 grid_a(n_chunks, s.n_kv_heads * 2, batch);
    enc_stats_kernel<<<grid_a, 256, 0, stream>>>(g, (const __half*)k_in, (const __half*)v_in, max_new, s.max_len,
                                                 seq_start, n_new, kv, vv, partial, ct, n_chunks, ws_b);
    if (g.dq) {
      const dim3 grid_r((max_new + 63) / 64, s.n_kv_heads * 2, batch);
      enc_brtn_kernel<<<grid_r, 64, 0, stream>>>(g, max_new, s.max_len, seq_start, n_new, kv, vv, ws_b);
    }
  }
  if (!freeze_means) {
    const int n_groups_new = s.group_size > 0 ? n_chunks : 1;
    const dim3 grid_m(n_groups_new, s.n_kv_heads * 2, batch);
    enc_means_kernel<<<grid_m, 128, 0, stream>>>(g, max_new, s.max_len, seq_start, n_new, kv, vv, partial, ct,
                                                 n_chunks);
  }
  const bool fused = freeze_means && !g.dq;  // the quantiser computes s1 itself (append mode)
  // 64 tokens per workgroup; calls that would leave most compute units idle use 16 (4 per wave)
  const int64_t blocks64 = (int64_t)((max_new + 63) / 64) * s.n_kv_heads * 2 * batch;
  const int wave_tokens = blocks64 >= 1024 ? 16 : 4;
  const dim3 grid_b((max_new + 4 * wave_tokens - 1) / (4 * wave_tokens), s.n_kv_heads * 2, batch);
  auto launch = [&](auto kernel) {
    kernel<<<grid_b, 256, 0, stream>>>(g, (const __half*)codebook, (const __half*)k_in, (const __half*)v_in, max_new,
                                       s.max_len, seq_start, n_new, kv, vv, wave_tokens, ws_b);
  };
  if (g.rope) {  // keys before the rotary embedding: matrix-core search only
    if (g.sign)
      fused ? launch(enc_quant_kernel<8, true, true, true, true>) : launch(enc_quant_kernel<8, true, false, true, true>);
    else if (s.sub_dim == 8)
      fused ? launch(enc_quant_kernel<8, true, true, false, true>) : launch(enc_quant_kernel<8, true, false, false, true>);
    else
      fused ? launch(enc_quant_kernel<4, true, true, false, true>) : launch(enc_quant_kernel<4, true, false, false, true>);
  } else if (g.sign) {
    if (use_mfma)
      fused ? launch(enc_quant_kernel<8, true, true, true>) : launch(enc_quant_kernel<8, true, false, true>);
    else
      fused ? launch(enc_quant_kernel<8, false, true, true>) : launch(enc_quant_kernel<8, false, false, true>);
  } else if (s.sub_dim == 8) {
    if (use_mfma)
      fused ? launch(enc_quant_kernel<8, true, true>) : launch(enc_quant_kernel<8, true, false>);
    else
      fused ? launch(enc_quant_kernel<8, false, true>) : launch(enc_quant_kernel<8, false, false>);
  } else {
    if (use_mfma)
      fused ? launch(enc_quant_kernel<4, true, true>) : launch(enc_quant_kernel<4, true, false>);
    else
      fused ? launch(enc_quant_kernel<4, false, true>) : launch(enc_quant_kernel<4, false, false>);
  }
  return hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
}

}  // namespace nsn
