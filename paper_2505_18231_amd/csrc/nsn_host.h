// Host-side glue shared by the translation units of libnsn.
#pragma once

#include "nsn_device.h"

namespace nsn {

// which formats keep their codes in the tiled layout (read by dec_tile_kernel)
inline bool shape_is_tiled(const nsn_shape& s) { return s.n_codes == kCodes && s.rope_table == nullptr; }

inline Geometry make_geometry(const nsn_shape& s) {
  Geometry g;
  g.dq = s.side_bits == 4;
  g.rope = static_cast<const unsigned char*>(s.rope_table);
  g.sign = s.n_codes == kSignCodes;
  g.tiled = shape_is_tiled(s);
  g.J = g.sign ? 2 * (s.head_dim / s.sub_dim) : s.head_dim / s.sub_dim;
  g.n_q_heads = s.n_q_heads;
  g.n_kv_heads = s.n_kv_heads;
  g.group_size = s.group_size;
  g.n_groups_max = s.group_size > 0 ? (s.max_len + s.group_size - 1) / s.group_size : 1;
  g.paged = s.page_size > 0;
  g.page_tokens = g.paged ? s.page_size : s.max_len;
  g.pages_per_seq = g.paged ? s.max_len / s.page_size : 1;
  auto log2_or_minus1 = [](int v) {
    if (v <= 0 || (v & (v - 1)) != 0) return -1;
    int k = 0;
    while ((1 << k) < v) ++k;
    return k;
  };
  g.group_shift = log2_or_minus1(s.group_size);
  g.page_shift = log2_or_minus1(g.page_tokens);
  return g;
}

inline CacheView make_view(const nsn_cache& c) {
  CacheView v;
  v.codes = c.codes;
  v.norms = static_cast<__half2*>(c.norms);
  v.means = static_cast<__half*>(c.means);
  v.block_table = c.block_table;
  return v;
}

void set_error(const char* fmt, ...);
int selected_variant(int op);  // NSN_VARIANT_* of NSN_OP_ENCODE / NSN_OP_DECODE (see nsn_select_variant)

// per-operation entry points implemented in the .hip files
size_t encode_workspace_bytes(const nsn_shape& s, int batch, int64_t max_new);
int encode_launch(const nsn_shape& s, const void* codebook, const void* k_in, const void* v_in, int max_new,
                  const int32_t* seq_start, const int32_t* n_new, int batch, int freeze_means,
                  const nsn_cache& kc, const nsn_cache& vc, void* workspace, hipStream_t stream);

// A resolved split count of kSplitsFlat selects the tiled-layout kernel's persistent instance: one workgroup
// per compute unit (at most kFlatRunsMax), each taking an equal run of the list of all 64-token groups.
constexpr int kSplitsFlat = 0;
constexpr int kFlatRunsMax = 256;
int decode_pick_splits(const nsn_shape& s, int batch, int max_seq_len, int requested);
bool decode_use_mfma(const nsn_shape& s);
int decode_mfma_splits(const nsn_shape& s, int batch, int max_seq_len, int requested);
size_t decode_mfma_workspace_bytes(const nsn_shape& s, int batch, int n_splits);
size_t decode_counter_bytes(const nsn_shape& s, int batch);  // arrival counters at the head of the decode workspace
int decode_tile_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                       const nsn_cache& vc, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                       int n_splits, void* workspace, size_t counter_bytes, const nsn_residual* residual, float* out,
                       hipStream_t stream);
int decode_mfma_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                       const nsn_cache& vc, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                       int n_splits, void* workspace, const nsn_residual* residual, float* out,
                       hipStream_t stream);
size_t decode_workspace_bytes(const nsn_shape& s, int batch, int n_splits);
int decode_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                  const nsn_cache& vc, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                  int n_splits, const nsn_residual* residual, float* out, void* workspace, hipStream_t stream);

int codebook_quantize(void* codebook_io, int sub_dim, uint8_t* codes_out, void* levels_out, hipStream_t stream);
size_t rope_table_bytes(int max_len);
int rope_table_build(const float* inv_freq_host, int max_len, void* table_dev, hipStream_t stream);

size_t codebook_workspace_bytes(int sub_dim, int64_t n_samples);
int codebook_run(const float* samples, int64_t n_samples, int sub_dim, int iters, void* codebook_out,
                 double* mse_host, void* workspace, hipStream_t stream);
int finetune_run(const float* samples, int64_t n_samples, int sub_dim, int iters, double lr, void* codebook_io,
                 double* cos_host, void* workspace, hipStream_t stream);

}  // namespace nsn
