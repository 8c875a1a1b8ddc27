// Cosine / sine table for keys that are normalised before the rotary embedding (Sec. 3.2 "NSN
// applied to key and value", App. B).  The angle of (position t, pair i) is t * inv_freq[i]; with
// t = 64 * block + j it is composed from a per-block and an in-block entry by the addition
// theorems, so no kernel evaluates a sine of a large argument itself.  Everything is evaluated in
// fp64 here, once.
#include "nsn_host.h"

namespace nsn {

struct InvFreq {
  float f[64];
};

// grid 64 + n_blk, block 64: workgroup r < 64 writes the in-block row j = r, the others one block row
__global__ __launch_bounds__(64) void rope_table_kernel(InvFreq inv, unsigned char* table) {
  const int i = threadIdx.x, r = blockIdx.x;
  const double theta = (double)inv.f[i];
  if (r < 64) {
    double s, c;
    sincos((double)r * theta, &s, &c);
    reinterpret_cast<double2*>(table + kRopeInOff)[r * 64 + i] = make_double2(c, s);
    const __half ch = f64_to_f16(c), sh = f64_to_f16(s);
    __half* hi = reinterpret_cast<__half*>(table + kRopeHiOff) + r * kHeadDim;
    __half* lo = reinterpret_cast<__half*>(table + kRopeLoOff) + r * kHeadDim;
    hi[i] = ch;
    hi[64 + i] = sh;
    lo[i] = f64_to_f16(c - (double)__half2float(ch));
    lo[64 + i] = f64_to_f16(s - (double)__half2float(sh));
  } else {
    const int blk = r - 64;
    double s, c;
    sincos((double)(64 * (int64_t)blk) * theta, &s, &c);
    unsigned char* rec = table + kRopeBlkOff + (int64_t)blk * kRopeBlkStride;
    reinterpret_cast<float2*>(rec)[i] = make_float2((float)c, (float)s);
    reinterpret_cast<double2*>(rec + kRopeBlk64)[i] = make_double2(c, s);
  }
}

size_t rope_table_bytes(int max_len) { return (size_t)kRopeBlkOff + (size_t)(max_len / 64) * kRopeBlkStride; }

int rope_table_build(const float* inv_freq_host, int max_len, void* table_dev, hipStream_t stream) {
  InvFreq inv;
  for (int i = 0; i < 64; ++i) inv.f[i] = inv_freq_host[i];
  const int n_blk = max_len / 64;
  rope_table_kernel<<<64 + n_blk, 64, 0, stream>>>(inv, static_cast<unsigned char*>(table_dev));
  return hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
}

}  // namespace nsn
