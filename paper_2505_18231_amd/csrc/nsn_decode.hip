// Decode attention over the coded cache (App. B): lookup-table form.
//
//   dec_lut_kernel    one workgroup per (split, query head, sequence): rotate q once, build the
//                     per-sub-vector q x codebook table in LDS, stream the split's tokens
//                     (gather-sum of table entries, rescale by the stored norms, add the
//                     q . mean term, online softmax, value accumulation in the rotated /
//                     codeword domain plus the mean-vector term) and emit an fp32 partial
//   dec_merge_kernel  merge the splits (running max / sum), one inverse Hadamard per head
#include <cstdlib>
#include <type_traits>

#include "nsn_host.h"

namespace nsn {

constexpr int kPartialStride = 2 * kHeadDim + 2;  // rotated acc, mean-term acc, m, l

__device__ inline float block_max_256(float v, float* red) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  const float r = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  return r;
}
__device__ inline float block_sum_256(float v, float* red) {
  v = xor_sum(v, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  const float r = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  return r;
}

// In-place Walsh-Hadamard transform of 128 floats in LDS by the first 64 threads of the block
// (unnormalised; all threads must call).
__device__ inline void fwht128_lds(float* x) {
  for (int s = 1; s < kHeadDim; s <<= 1) {
    __syncthreads();
    if (threadIdx.x < 64) {
      const int i = ((threadIdx.x & ~(s - 1)) << 1) | (threadIdx.x & (s - 1));
      const float a = x[i], b = x[i + s];
      x[i] = a + b;
      x[i + s] = a - b;
    }
  }
  __syncthreads();
}

template <int SUB>
__global__ __launch_bounds__(256) void dec_lut_kernel(Geometry g, const __half* __restrict__ codebook,
                                                      const __half* __restrict__ q, CacheView kc, CacheView vc,
                                                      const int32_t* __restrict__ seq_lens, float scale,
                                                      int n_splits, float* __restrict__ partial) {
  constexpr int J = kHeadDim / SUB;
  constexpr int TS = 256 / J;  // token sub-groups of the value phase
  __shared__ float lut[J][kCodes];
  __shared__ float cb[kCodes][SUB];
  __shared__ float qs[kHeadDim], qh[kHeadDim];
  __shared__ float pa[256], pb[256];
  __shared__ float red[4], qo_s[4], beta_s[4];
  __shared__ float accred[TS][kHeadDim];

  const int split = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int h = hq / (g.n_q_heads / g.n_kv_heads);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int len = seq_lens[b];
  const int per = (((len + n_splits - 1) / n_splits) + 63) & ~63;
  const int t0 = split * per, t1 = min(len, t0 + per);
  float* P = partial + ((int64_t)(b * g.n_q_heads + hq) * n_splits + split) * kPartialStride;
  if (t0 >= t1) {  // empty split (uniform for the block)
    if (tid < kHeadDim) {
      P[tid] = 0.f;
      P[kHeadDim + tid] = 0.f;
    }
    if (tid == 0) {
      P[2 * kHeadDim] = -INFINITY;
      P[2 * kHeadDim + 1] = 0.f;
    }
    return;
  }

  // d1: rotate the query once
  if (tid < kHeadDim) {
    const float v = __half2float(q[(int64_t)(b * g.n_q_heads + hq) * kHeadDim + tid]);
    qs[tid] = v;
    qh[tid] = v;
  }
  for (int i = tid; i < kCodes * SUB; i += 256) cb[i / SUB][i % SUB] = __half2float(codebook[i]);
  fwht128_lds(qh);
  // d2: table LUT[j][c] = q_Had[j-th sub-vector] . C[c]
  {
    const int c = tid;
    float cw[SUB];
#pragma unroll
    for (int i = 0; i < SUB; ++i) cw[i] = cb[c][i];
    for (int j = 0; j < J; ++j) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < SUB; ++i) s = fmaf(qh[j * SUB + i], cw[i], s);
      lut[j][c] = s * (float)kInvSqrtD;
    }
  }
  __syncthreads();

  const int64_t mean_base = (int64_t)(b * g.n_kv_heads + h) * g.n_groups_max;
  const int jv = tid % J, ts = tid / J;
  float m_run = -INFINITY, l_run = 0.f, accm = 0.f;
  float acc[SUB];
#pragma unroll
  for (int i = 0; i < SUB; ++i) acc[i] = 0.f;

  for (int c0 = t0; c0 < t1; c0 += 256) {
    const int g_first = group_of(g, c0);
    const int n_g = group_of(g, min(c0 + 255, t1 - 1)) - g_first + 1;  // <= 4
    if (wave < n_g) {  // q . o^k of the groups this chunk touches
      const __half2 o2 =
          *reinterpret_cast<const __half2*>(kc.means + (mean_base + g_first + wave) * kHeadDim + 2 * lane);
      float d = qs[2 * lane] * __low2float(o2) + qs[2 * lane + 1] * __high2float(o2);
      d = xor_sum(d, 64);
      if (lane == 0) qo_s[wave] = d;
    }
    __syncthreads();

    // d3: score of this thread's token
    const int t = c0 + tid;
    const bool valid = t < t1;
    float score = -INFINITY, av = 0.f, bv = 0.f;
    if (valid) {
      const int64_t base = unit_token_base(g, kc.block_table, b, h, t);
      const int tin = token_in_unit(g, t);
      float sum = 0.f;
      if (g.tiled) {  // a token's J bytes lie in four runs of J / 4 (one per 32-channel quarter)
        constexpr int QS = J / 4;
        typedef typename std::conditional<QS == 8, uint2, uint32_t>::type run_t;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const run_t run = *reinterpret_cast<const run_t*>(kc.codes + base * J + k_code_offset_tiled(J, tin, c * QS));
          uint32_t wds[2] = {0u, 0u};
          if constexpr (QS == 8)
            wds[0] = run.x, wds[1] = run.y;
          else
            wds[0] = run;
#pragma unroll
          for (int e = 0; e < QS; ++e) sum += lut[c * QS + e][(wds[e >> 2] >> ((e & 3) * 8)) & 0xff];
        }
      } else {
        const uint4* kp = reinterpret_cast<const uint4*>(kc.codes + (base + tin) * J);
#pragma unroll
        for (int w4 = 0; w4 < J / 16; ++w4) {
          const uint4 cw = kp[w4];
          const uint32_t wds[4] = {cw.x, cw.y, cw.z, cw.w};
#pragma unroll
          for (int e = 0; e < 16; ++e) sum += lut[w4 * 16 + e][(wds[e >> 2] >> ((e & 3) * 8)) & 0xff];
        }
      }
      const __half2 nk = kc.norms[base + tin];
      score = scale * (__low2float(nk) * sum + __high2float(nk) * qo_s[group_of(g, t) - g_first]);
      const int64_t vbase = unit_token_base(g, vc.block_table, b, h, t);
      const __half2 nv = vc.norms[vbase + tin];
      av = __low2float(nv);
      bv = __high2float(nv);
    }
    // d4: online softmax
    const float cmax = block_max_256(score, red);
    const float m_new = fmaxf(m_run, cmax);
    const float corr = __expf(m_run - m_new);  // 0 on the first chunk
    const float p = valid ? __expf(score - m_new) : 0.f;
    const float psum = block_sum_256(p, red);
    l_run = l_run * corr + psum;
    m_run = m_new;
    pa[tid] = p * av;
    pb[tid] = p * bv;
    __syncthreads();

    // d5: value accumulation in the rotated domain: lane owns sub-vector jv of tokens ts, ts+TS, ..
#pragma unroll
    for (int i = 0; i < SUB; ++i) acc[i] *= corr;
    for (int tt = ts; tt < 256; tt += TS) {
      const int tv = c0 + tt;
      if (tv >= t1) break;
      const int64_t vbase = unit_token_base(g, vc.block_table, b, h, tv);
      const int tin = token_in_unit(g, tv);
      const int code = vc.codes[vbase * J + code_offset(g.tiled, true, J, tin, jv)];
      const float w = pa[tt];
#pragma unroll
      for (int i = 0; i < SUB; ++i) acc[i] = fmaf(w, cb[code][i], acc[i]);
    }
    // mean-vector term: beta_g = sum_{t in g} p_t b^v_t, then += beta_g * o^v_g
    if (wave < n_g) {
      float s = 0.f;
      for (int tt = lane; tt < 256; tt += 64) {
        const int tv = c0 + tt;
        if (tv < t1 && group_of(g, tv) == g_first + wave) s += pb[tt];
      }
      s = xor_sum(s, 64);
      if (lane == 0) beta_s[wave] = s;
    }
    __syncthreads();
    if (tid < kHeadDim) {
      accm *= corr;
      for (int w = 0; w < n_g; ++w)
        accm = fmaf(beta_s[w], __half2float(vc.means[(mean_base + g_first + w) * kHeadDim + tid]), accm);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < SUB; ++i) accred[ts][jv * SUB + i] = acc[i];
  __syncthreads();
  if (tid < kHeadDim) {
    float s = 0.f;
    for (int k = 0; k < TS; ++k) s += accred[k][tid];
    P[tid] = s;
    P[kHeadDim + tid] = accm;
  }
  if (tid == 0) {
    P[2 * kHeadDim] = m_run;
    P[2 * kHeadDim + 1] = l_run;
  }
}

// d6: merge the splits of one (sequence, query head) and undo the rotation once.
__global__ __launch_bounds__(128) void dec_merge_kernel(int n_q_heads, int n_splits,
                                                        const float* __restrict__ partial,
                                                        float* __restrict__ out) {
  __shared__ float rot[kHeadDim];
  const int hq = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  const float* P = partial + (int64_t)(b * n_q_heads + hq) * n_splits * kPartialStride;
  float M = -INFINITY;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, P[s * kPartialStride + 2 * kHeadDim]);
  float L = 0.f, r = 0.f, mm = 0.f;
  if (M > -INFINITY) {
    for (int s = 0; s < n_splits; ++s) {
      const float* ps = P + s * kPartialStride;
      const float e = __expf(ps[2 * kHeadDim] - M);
      L = fmaf(e, ps[2 * kHeadDim + 1], L);
      r = fmaf(e, ps[c], r);
      mm = fmaf(e, ps[kHeadDim + c], mm);
    }
  }
  rot[c] = r;
  for (int s = 1; s < kHeadDim; s <<= 1) {
    __syncthreads();
    if (c < 64) {
      const int i = ((c & ~(s - 1)) << 1) | (c & (s - 1));
      const float a0 = rot[i], a1 = rot[i + s];
      rot[i] = a0 + a1;
      rot[i + s] = a0 - a1;
    }
  }
  __syncthreads();
  out[(int64_t)(b * n_q_heads + hq) * kHeadDim + c] = (L > 0.f) ? (rot[c] * (float)kInvSqrtD + mm) / L : 0.f;
}

// ---------------------------------------------------------------------------------------
bool decode_use_mfma(const nsn_shape& s) {
  if (s.n_codes == kSignCodes) return true;   // the sign + index format exists in the matrix-core kernel only
  // up to 8 query heads per kv head (checked with the shape): one launch per four heads
  return selected_variant(NSN_OP_DECODE) != NSN_VARIANT_ALT;  // the alternative is the lookup-table kernel
}

int decode_pick_splits(const nsn_shape& s, int batch, int max_seq_len, int requested) {
  if (decode_use_mfma(s)) return decode_mfma_splits(s, batch, max_seq_len, requested);
  const int cap = max(1, min(64, (max_seq_len + 255) / 256));
  if (requested > 0) return min(requested, 64);
  const int rows = max(1, batch * s.n_q_heads);
  return max(1, min(cap, (1024 + rows - 1) / rows));
}

size_t decode_workspace_bytes(const nsn_shape& s, int batch, int n_splits) {
  if (decode_use_mfma(s)) return decode_mfma_workspace_bytes(s, batch, n_splits);
  return (size_t)batch * s.n_q_heads * n_splits * kPartialStride * sizeof(float);
}

int decode_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                  const nsn_cache& vc, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                  int n_splits, const nsn_residual* residual, float* out, void* workspace, hipStream_t stream) {
  if (decode_use_mfma(s)) {
    const int rc = decode_mfma_launch(s, codebook, q, kc, vc, seq_lens, batch, max_seq_len, scale, n_splits,
                                      workspace, residual, out, stream);
    return rc != NSN_OK ? rc : hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
  }
  if (residual) return NSN_ERR_UNSUPPORTED;  // the lookup-table kernel reads coded tokens only
  const Geometry g = make_geometry(s);
  const CacheView kv = make_view(kc), vv = make_view(vc);
  float* partial = static_cast<float*>(workspace);
  const dim3 grid(n_splits, s.n_q_heads, batch);
  if (s.sub_dim == 8)
    dec_lut_kernel<8><<<grid, 256, 0, stream>>>(g, (const __half*)codebook, (const __half*)q, kv, vv, seq_lens,
                                                scale, n_splits, partial);
  else
    dec_lut_kernel<4><<<grid, 256, 0, stream>>>(g, (const __half*)codebook, (const __half*)q, kv, vv, seq_lens,
                                                scale, n_splits, partial);
  dec_merge_kernel<<<dim3(s.n_q_heads, batch), 128, 0, stream>>>(s.n_q_heads, n_splits, partial, out);
  return hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
}

}  // namespace nsn
