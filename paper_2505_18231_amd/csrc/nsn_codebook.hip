// K-Means codebook on standard-normal samples (Sec. 3.4, the K-Means baseline) and its
// fine-tuning for cosine distance.
//
// Lloyd iterations entirely on the device, deterministic (no atomics):
//   km_assign_kernel  nearest centroid per sample (same fp32-scan + fp64-recheck search as the
//                     encoder), per-block fp64 error sums
//   km_update_kernel  one workgroup per cluster: fp64 mean of its members, fixed reduction order;
//                     an empty cluster keeps its centroid
#include "nsn_host.h"
#include "nsn_vq.h"

namespace nsn {

constexpr int kAssignBlocks = 1024;

__global__ void km_init_kernel(const float* __restrict__ samples, double* __restrict__ centroids, int n_elems) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_elems) centroids[i] = (double)samples[i];
}

__global__ void km_round_kernel(double* __restrict__ centroids, __half* __restrict__ out, int n_elems) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_elems) {
    const __half hv = f64_to_f16(centroids[i]);
    out[i] = hv;
    centroids[i] = (double)__half2float(hv);
  }
}

template <int SUB>
__global__ __launch_bounds__(256) void km_assign_kernel(const float* __restrict__ samples, int64_t n,
                                                        const double* __restrict__ centroids,
                                                        uint8_t* __restrict__ assign,
                                                        double* __restrict__ block_err) {
  __shared__ VqTables<SUB> T;
  __shared__ double red[4];
  vq_tables_fill<SUB>(T, [&](int c, int i) { return centroids[c * SUB + i]; });
  double err = 0.0;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * 256) {
    double y[SUB];
#pragma unroll
    for (int i = 0; i < SUB; ++i) y[i] = (double)samples[idx * SUB + i];
    const int code = vq_search<SUB>(T, y);
    assign[idx] = (uint8_t)code;
    err += exact_dist<SUB>(T, y, code);
  }
  err = xor_sum(err, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = err;
  __syncthreads();
  if (threadIdx.x == 0) block_err[blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
}

constexpr int kUpdateThreads = 1024;
constexpr int kUpdateWaves = kUpdateThreads / 64;

// Calls fn(idx) for every sample assigned to cluster k, in an order that depends only on n and
// the workgroup size (by thread, then ascending index), so the fp64 sums that follow are
// reproducible.  The assignments are scanned 16 to a load, four loads in flight; a word is taken
// apart only if one of its four bytes matches.
template <class F>
__device__ __forceinline__ void for_each_member(const uint8_t* __restrict__ assign, int64_t n, int k, F&& fn) {
  constexpr int64_t kStep = (int64_t)kUpdateThreads * 16;
  const int64_t n16 = n & ~(int64_t)15;
  const uint32_t kk = (uint32_t)k * 0x01010101u;
  for (int64_t base = (int64_t)threadIdx.x * 16; base < n16; base += 4 * kStep) {
    uint4 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      w[u] = base + u * kStep < n16 ? *reinterpret_cast<const uint4*>(assign + base + u * kStep)
                                    : make_uint4(~kk, ~kk, ~kk, ~kk);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t ws[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t x = ws[j] ^ kk;  // a zero byte marks a member
        if (((x - 0x01010101u) & ~x & 0x80808080u) != 0u) {
#pragma unroll
          for (int b = 0; b < 4; ++b)
            if (((x >> (8 * b)) & 0xffu) == 0u) fn(base + u * kStep + 4 * j + b);
        }
      }
    }
  }
  for (int64_t idx = n16 + threadIdx.x; idx < n; idx += kUpdateThreads)
    if (assign[idx] == k) fn(idx);
}

template <int SUB>
__global__ __launch_bounds__(kUpdateThreads) void km_update_kernel(const float* __restrict__ samples, int64_t n,
                                                        const uint8_t* __restrict__ assign,
                                                        double* __restrict__ centroids) {
  __shared__ double red[kUpdateWaves][SUB + 1];
  const int k = blockIdx.x;
  double sum[SUB];
#pragma unroll
  for (int i = 0; i < SUB; ++i) sum[i] = 0.0;
  double cnt = 0.0;
  for_each_member(assign, n, k, [&](int64_t idx) {
#pragma unroll
    for (int i = 0; i < SUB; ++i) sum[i] += (double)samples[idx * SUB + i];
    cnt += 1.0;
  });
#pragma unroll
  for (int i = 0; i < SUB; ++i) sum[i] = xor_sum(sum[i], 64);
  cnt = xor_sum(cnt, 64);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int i = 0; i < SUB; ++i) red[wave][i] = sum[i];
    red[wave][SUB] = cnt;
  }
  __syncthreads();
  if (threadIdx.x <= SUB) {
    const int i = threadIdx.x;
    double tot_cnt = 0.0, tot = 0.0;
    for (int w = 0; w < kUpdateWaves; ++w) {
      tot_cnt += red[w][SUB];
      tot += red[w][i];  // for i == SUB the count again: unused
    }
    if (i < SUB && tot_cnt > 0.0) centroids[k * SUB + i] = tot / tot_cnt;
  }
}

// Fine-tuning for cosine distance (Sec. 3.4): one workgroup per codeword sums x / |x| over its
// samples in a fixed order (fp64), then moves the codeword along the part of that sum that is
// orthogonal to it:  c += lr / (N |c|) * (S - (S . c^) c^).   cos_sum[k] = S . c^ is the cluster's
// share of the summed cosine similarity BEFORE the move.
template <int SUB>
__global__ __launch_bounds__(kUpdateThreads) void ft_update_kernel(const float* __restrict__ samples, int64_t n,
                                                        const uint8_t* __restrict__ assign,
                                                        double* __restrict__ centroids, double lr,
                                                        double* __restrict__ cos_sum) {
  __shared__ double red[kUpdateWaves][SUB];
  const int k = blockIdx.x;
  double sum[SUB];
#pragma unroll
  for (int i = 0; i < SUB; ++i) sum[i] = 0.0;
  for_each_member(assign, n, k, [&](int64_t idx) {
    double x[SUB], n2 = 0.0;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      x[i] = (double)samples[idx * SUB + i];
      n2 += x[i] * x[i];
    }
    if (n2 > 0.0) {
      const double nx = sqrt(n2);
#pragma unroll
      for (int i = 0; i < SUB; ++i) sum[i] += x[i] / nx;
    }
  });
#pragma unroll
  for (int i = 0; i < SUB; ++i) sum[i] = xor_sum(sum[i], 64);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int i = 0; i < SUB; ++i) red[wave][i] = sum[i];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double S[SUB], c[SUB], cn2 = 0.0;
#pragma unroll
    for (int i = 0; i < SUB; ++i) {
      S[i] = 0.0;
      for (int w = 0; w < kUpdateWaves; ++w) S[i] += red[w][i];
      c[i] = centroids[k * SUB + i];
      cn2 += c[i] * c[i];
    }
    double along = 0.0;
    if (cn2 > 0.0) {
      const double cn = sqrt(cn2);
#pragma unroll
      for (int i = 0; i < SUB; ++i) along += S[i] * (c[i] / cn);
#pragma unroll
      for (int i = 0; i < SUB; ++i)
        centroids[k * SUB + i] = c[i] + lr * ((S[i] - along * (c[i] / cn)) / ((double)n * cn));
    }
    cos_sum[k] = along;
  }
}

__global__ void ft_load_kernel(const __half* __restrict__ in, double* __restrict__ centroids, int n_elems) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_elems) centroids[i] = (double)__half2float(in[i]);
}

size_t codebook_workspace_bytes(int sub_dim, int64_t n_samples) {
  return (size_t)kCodes * sub_dim * sizeof(double) + kAssignBlocks * sizeof(double) + kCodes * sizeof(double) +
         (size_t)((n_samples + 255) / 256) * 256;
}

template <int SUB>
static int codebook_run_t(const float* samples, int64_t n, int iters, void* codebook_out, double* mse_host,
                          void* workspace, hipStream_t stream) {
  double* centroids = static_cast<double*>(workspace);
  double* block_err = centroids + kCodes * SUB;
  uint8_t* assign = reinterpret_cast<uint8_t*>(block_err + kAssignBlocks + kCodes);
  const int n_elems = kCodes * SUB;
  km_init_kernel<<<(n_elems + 255) / 256, 256, 0, stream>>>(samples, centroids, n_elems);
  for (int it = 0; it < iters; ++it) {
    km_assign_kernel<SUB><<<kAssignBlocks, 256, 0, stream>>>(samples, n, centroids, assign, block_err);
    km_update_kernel<SUB><<<kCodes, kUpdateThreads, 0, stream>>>(samples, n, assign, centroids);
  }
  km_round_kernel<<<(n_elems + 255) / 256, 256, 0, stream>>>(centroids, static_cast<__half*>(codebook_out), n_elems);
  km_assign_kernel<SUB><<<kAssignBlocks, 256, 0, stream>>>(samples, n, centroids, assign, block_err);
  if (hipGetLastError() != hipSuccess) return NSN_ERR_HIP;
  double host_err[kAssignBlocks];
  if (hipMemcpyAsync(host_err, block_err, sizeof(host_err), hipMemcpyDeviceToHost, stream) != hipSuccess)
    return NSN_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return NSN_ERR_HIP;
  if (mse_host) {
    double tot = 0.0;
    for (int i = 0; i < kAssignBlocks; ++i) tot += host_err[i];
    *mse_host = tot / ((double)n * SUB);
  }
  return NSN_OK;
}

template <int SUB>
static int finetune_run_t(const float* samples, int64_t n, int iters, double lr, void* codebook_io, double* cos_host,
                          void* workspace, hipStream_t stream) {
  double* centroids = static_cast<double*>(workspace);
  double* block_err = centroids + kCodes * SUB;
  double* cos_sum = block_err + kAssignBlocks;
  uint8_t* assign = reinterpret_cast<uint8_t*>(cos_sum + kCodes);
  const int n_elems = kCodes * SUB;
  double host_cos[kCodes];
  auto mean_cos = [&](double* out) -> int {  // assignment + cosine sums of the current centroids (no move: lr = 0)
    km_assign_kernel<SUB><<<kAssignBlocks, 256, 0, stream>>>(samples, n, centroids, assign, block_err);
    ft_update_kernel<SUB><<<kCodes, kUpdateThreads, 0, stream>>>(samples, n, assign, centroids, 0.0, cos_sum);
    if (hipGetLastError() != hipSuccess) return NSN_ERR_HIP;
    if (hipMemcpyAsync(host_cos, cos_sum, sizeof(host_cos), hipMemcpyDeviceToHost, stream) != hipSuccess)
      return NSN_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return NSN_ERR_HIP;
    double tot = 0.0;
    for (int k = 0; k < kCodes; ++k) tot += host_cos[k];
    *out = tot / (double)n;
    return NSN_OK;
  };
  ft_load_kernel<<<(n_elems + 255) / 256, 256, 0, stream>>>(static_cast<const __half*>(codebook_io), centroids, n_elems);
  int rc = NSN_OK;
  double before = 0.0, after = 0.0;
  if (cos_host && (rc = mean_cos(&before)) != NSN_OK) return rc;
  for (int it = 0; it < iters; ++it) {
    km_assign_kernel<SUB><<<kAssignBlocks, 256, 0, stream>>>(samples, n, centroids, assign, block_err);
    ft_update_kernel<SUB><<<kCodes, kUpdateThreads, 0, stream>>>(samples, n, assign, centroids, lr, cos_sum);
  }
  km_round_kernel<<<(n_elems + 255) / 256, 256, 0, stream>>>(centroids, static_cast<__half*>(codebook_io), n_elems);
  if (hipGetLastError() != hipSuccess) return NSN_ERR_HIP;
  if (cos_host) {
    if ((rc = mean_cos(&after)) != NSN_OK) return rc;
    cos_host[0] = before;
    cos_host[1] = after;
  } else if (hipStreamSynchronize(stream) != hipSuccess) {
    return NSN_ERR_HIP;
  }
  return NSN_OK;
}

int finetune_run(const float* samples, int64_t n_samples, int sub_dim, int iters, double lr, void* codebook_io,
                 double* cos_host, void* workspace, hipStream_t stream) {
  return sub_dim == 8 ? finetune_run_t<8>(samples, n_samples, iters, lr, codebook_io, cos_host, workspace, stream)
                      : finetune_run_t<4>(samples, n_samples, iters, lr, codebook_io, cos_host, workspace, stream);
}

int codebook_run(const float* samples, int64_t n_samples, int sub_dim, int iters, void* codebook_out,
                 double* mse_host, void* workspace, hipStream_t stream) {
  return sub_dim == 8 ? codebook_run_t<8>(samples, n_samples, iters, codebook_out, mse_host, workspace, stream)
                      : codebook_run_t<4>(samples, n_samples, iters, codebook_out, mse_host, workspace, stream);
}

// Codebook entries on 16 levels (Sec. 3.5): one workgroup; thread c owns codeword c.
template <int SUB>
__global__ __launch_bounds__(256) void cb_quantize_kernel(__half* __restrict__ codebook, uint8_t* __restrict__ codes,
                                                          __half* __restrict__ levels) {
  __shared__ float red_lo[4], red_hi[4];
  const int c = threadIdx.x, lane = c & 63, wave = c >> 6;
  float x[SUB], lo = INFINITY, hi = -INFINITY;
#pragma unroll
  for (int i = 0; i < SUB; ++i) {
    x[i] = __half2float(codebook[c * SUB + i]);
    lo = fminf(lo, x[i]);
    hi = fmaxf(hi, x[i]);
  }
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    lo = fminf(lo, __shfl_xor(lo, m, 64));
    hi = fmaxf(hi, __shfl_xor(hi, m, 64));
  }
  if (lane == 0) red_lo[wave] = lo, red_hi[wave] = hi;
  __syncthreads();
  lo = fminf(fminf(red_lo[0], red_lo[1]), fminf(red_lo[2], red_lo[3]));
  hi = fmaxf(fmaxf(red_hi[0], red_hi[1]), fmaxf(red_hi[2], red_hi[3]));
  const __half mn16 = f64_to_f16((double)lo), st16 = f64_to_f16(((double)hi - (double)lo) / 15.0);
  const double mn = (double)__half2float(mn16), st = (double)__half2float(st16);
#pragma unroll
  for (int i = 0; i < SUB; ++i) {
    int code = 0;
    if (st != 0.0) code = (int)fmin(fmax(floor(((double)x[i] - mn) / st + 0.5), 0.0), 15.0);
    codebook[c * SUB + i] = f64_to_f16(mn + st * (double)code);
    if (codes) codes[c * SUB + i] = (uint8_t)code;
  }
  if (levels && c == 0) levels[0] = mn16, levels[1] = st16;
}

int codebook_quantize(void* codebook_io, int sub_dim, uint8_t* codes_out, void* levels_out, hipStream_t stream) {
  if (sub_dim == 4)
    cb_quantize_kernel<4><<<1, 256, 0, stream>>>(static_cast<__half*>(codebook_io), codes_out, static_cast<__half*>(levels_out));
  else
    cb_quantize_kernel<8><<<1, 256, 0, stream>>>(static_cast<__half*>(codebook_io), codes_out, static_cast<__half*>(levels_out));
  return hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
}

}  // namespace nsn
