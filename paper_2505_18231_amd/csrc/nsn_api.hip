// extern "C" boundary of libnsn: argument validation and dispatch only.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "nsn_host.h"

namespace nsn {

static thread_local char g_err[256] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

// kernel variant per operation (encode, decode); the environment gives the initial value, once
static std::atomic<int>* variants() {
  static std::atomic<int> v[2];
  static const bool init = [] {
    const char* e = getenv("NSN_ENCODE_IMPL");
    const char* d = getenv("NSN_DECODE_IMPL");
    v[NSN_OP_ENCODE].store(e && e[0] == 'v' ? NSN_VARIANT_ALT : NSN_VARIANT_DEFAULT);
    v[NSN_OP_DECODE].store(d && d[0] == 'l' ? NSN_VARIANT_ALT : NSN_VARIANT_DEFAULT);
    return true;
  }();
  (void)init;
  return v;
}

int selected_variant(int op) { return variants()[op].load(std::memory_order_relaxed); }

static int check_shape(const nsn_shape* s) {
  if (!s) {
    set_error("shape is NULL");
    return NSN_ERR_INVALID_ARG;
  }
  const bool plain = s->n_codes == kCodes && (s->sub_dim == 4 || s->sub_dim == 8);
  const bool sign = s->n_codes == kSignCodes && s->sub_dim == 8;
  if (s->head_dim != kHeadDim || !(plain || sign)) {
    set_error("unsupported shape: head_dim=%d (128), n_codes=%d (256, or 65536 = sign + index with sub_dim 8), "
              "sub_dim=%d (4 or 8)", s->head_dim, s->n_codes, s->sub_dim);
    return NSN_ERR_UNSUPPORTED;
  }
  if (s->n_kv_heads <= 0 || s->n_q_heads <= 0 || s->n_q_heads % s->n_kv_heads != 0) {
    set_error("n_q_heads=%d must be a positive multiple of n_kv_heads=%d", s->n_q_heads, s->n_kv_heads);
    return NSN_ERR_INVALID_ARG;
  }
  if (s->n_q_heads / s->n_kv_heads > 8) {
    set_error("more than 8 query heads per kv head is not supported");
    return NSN_ERR_UNSUPPORTED;
  }
  if (s->group_size < 0 || s->group_size % 64 != 0) {
    set_error("group_size=%d must be 0 or a multiple of 64", s->group_size);
    return NSN_ERR_INVALID_ARG;
  }
  if (s->max_len <= 0 || s->max_len % 64 != 0) {
    set_error("max_len=%d must be a positive multiple of 64", s->max_len);
    return NSN_ERR_INVALID_ARG;
  }
  if (s->side_bits != 0 && s->side_bits != 16 && s->side_bits != 4) {
    set_error("side_bits=%d must be 16 (or 0) or 4", s->side_bits);
    return NSN_ERR_UNSUPPORTED;
  }
  if (s->rope_table && (reinterpret_cast<uintptr_t>(s->rope_table) & 255) != 0) {
    set_error("rope_table must be 256-byte aligned");
    return NSN_ERR_INVALID_ARG;
  }
  if (s->page_size < 0 || s->page_size % 64 != 0 || (s->page_size > 0 && s->max_len % s->page_size != 0)) {
    set_error("page_size=%d must be 0 or a multiple of 64 dividing max_len=%d", s->page_size, s->max_len);
    return NSN_ERR_INVALID_ARG;
  }
  return NSN_OK;
}

static int check_cache(const nsn_shape* s, const nsn_cache* c, const char* name) {
  if (!c || !c->codes || !c->norms || !c->means) {
    set_error("%s cache or one of its pointers is NULL", name);
    return NSN_ERR_INVALID_ARG;
  }
  if (s->page_size > 0 && !c->block_table) {
    set_error("%s cache: paged layout needs a block_table", name);
    return NSN_ERR_INVALID_ARG;
  }
  return NSN_OK;
}

// ---- scratch of nsn_decode_attention_noalloc ---------------------------------------------------
// A fixed array in the library's device image takes the place of the caller's workspace (arrival
// counters + split partials).  Every GPU that loads the library holds its own copy; the array's name is
// only a host-side handle, its device address comes from hipGetSymbolAddress once per device.
constexpr size_t kScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (nullptr + error text on failure)
static void* scratch_address() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("decode (noalloc): no current device, or device index beyond %d", kMaxDevices - 1);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      set_error("decode (noalloc): hipGetSymbolAddress failed: %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// the arrival counters must start at zero (a fill kernel, not a memset node: the call may be captured)
__global__ void scratch_clear_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace nsn

using namespace nsn;

extern "C" {

int64_t nsn_k_code_offset(const nsn_shape* shape, int64_t t, int j) {
  if (check_shape(shape) != NSN_OK) return -1;
  const Geometry g = make_geometry(*shape);
  return (t < 0 || j < 0 || j >= g.J) ? -1 : code_offset(g.tiled, false, g.J, t, j);
}
int64_t nsn_v_code_offset(const nsn_shape* shape, int64_t t, int j) {
  if (check_shape(shape) != NSN_OK) return -1;
  const Geometry g = make_geometry(*shape);
  return (t < 0 || j < 0 || j >= g.J) ? -1 : code_offset(g.tiled, true, g.J, t, j);
}

int nsn_max_groups(const nsn_shape* shape) {
  if (check_shape(shape) != NSN_OK) return 0;
  return make_geometry(*shape).n_groups_max;
}

const char* nsn_last_error(void) { return g_err; }

int nsn_select_variant(int op, int variant) {
  if ((op != NSN_OP_ENCODE && op != NSN_OP_DECODE) || (variant != NSN_VARIANT_DEFAULT && variant != NSN_VARIANT_ALT)) {
    set_error("select_variant: op must be NSN_OP_ENCODE or NSN_OP_DECODE, variant NSN_VARIANT_DEFAULT or NSN_VARIANT_ALT");
    return NSN_ERR_INVALID_ARG;
  }
  return variants()[op].exchange(variant);
}

size_t nsn_rope_table_bytes(int max_len) {
  return (max_len > 0 && max_len % 64 == 0) ? rope_table_bytes(max_len) : 0;
}

int nsn_build_rope_table(const float* inv_freq_host, int max_len, void* table_dev, size_t table_bytes,
                         void* stream) {
  if (!inv_freq_host || !table_dev || max_len <= 0 || max_len % 64 != 0 ||
      (reinterpret_cast<uintptr_t>(table_dev) & 255) != 0 || table_bytes < rope_table_bytes(max_len)) {
    set_error("build_rope_table: null pointer, max_len=%d not a positive multiple of 64, table not 256-byte aligned "
              "or smaller than %zu bytes", max_len, max_len > 0 ? rope_table_bytes(max_len) : (size_t)0);
    return NSN_ERR_INVALID_ARG;
  }
  const int rc = rope_table_build(inv_freq_host, max_len, table_dev, static_cast<hipStream_t>(stream));
  if (rc == NSN_ERR_HIP) set_error("build_rope_table: launch failed: %s", hipGetErrorString(hipGetLastError()));
  return rc;
}

size_t nsn_workspace_bytes(const nsn_shape* shape, int op, int batch, int64_t n, int n_splits) {
  if (op == NSN_OP_CODEBOOK) {
    if (!shape || (shape->sub_dim != 4 && shape->sub_dim != 8) || n <= 0) return 0;
    return codebook_workspace_bytes(shape->sub_dim, n);
  }
  if (check_shape(shape) != NSN_OK || batch <= 0) return 0;
  if (op == NSN_OP_ENCODE) return n > 0 ? encode_workspace_bytes(*shape, batch, n) : 0;
  if (op == NSN_OP_DECODE)
    return decode_workspace_bytes(*shape, batch, decode_pick_splits(*shape, batch, shape->max_len, n_splits));
  return 0;
}

int nsn_build_codebook(const float* samples_dev, int64_t n_samples, int sub_dim, int n_codes, int iters,
                       void* codebook_dev, double* mse_host, void* workspace, size_t workspace_bytes,
                       void* stream) {
  if (n_codes != kCodes || (sub_dim != 4 && sub_dim != 8)) {
    set_error("unsupported codebook: n_codes=%d (256), sub_dim=%d (4 or 8)", n_codes, sub_dim);
    return NSN_ERR_UNSUPPORTED;
  }
  if (!samples_dev || !codebook_dev || n_samples < n_codes || iters < 0) {
    set_error("build_codebook: null pointer, n_samples=%lld < n_codes, or iters=%d < 0", (long long)n_samples,
              iters);
    return NSN_ERR_INVALID_ARG;
  }
  if (!workspace || workspace_bytes < codebook_workspace_bytes(sub_dim, n_samples)) {
    set_error("build_codebook: workspace of %zu bytes needed", codebook_workspace_bytes(sub_dim, n_samples));
    return NSN_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 15) {
    set_error("build_codebook: the workspace must start on a 16-byte boundary");
    return NSN_ERR_INVALID_ARG;
  }
  const int rc = codebook_run(samples_dev, n_samples, sub_dim, iters, codebook_dev, mse_host, workspace,
                              static_cast<hipStream_t>(stream));
  if (rc == NSN_ERR_HIP) set_error("build_codebook: HIP error: %s", hipGetErrorString(hipGetLastError()));
  return rc;
}

int nsn_finetune_codebook(const float* samples_dev, int64_t n_samples, int sub_dim, int n_codes, int iters,
                          double lr, void* codebook_dev, double* cos_host, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (n_codes != 256 || (sub_dim != 4 && sub_dim != 8)) {
    set_error("finetune_codebook: unsupported n_codes=%d sub_dim=%d (256 codes of 4 or 8 dims)", n_codes, sub_dim);
    return NSN_ERR_UNSUPPORTED;
  }
  if (!samples_dev || !codebook_dev || n_samples < 1 || iters < 0 || !(lr >= 0.0)) {
    set_error("finetune_codebook: null pointer, n_samples=%lld < 1, iters=%d < 0 or a negative rate",
              (long long)n_samples, iters);
    return NSN_ERR_INVALID_ARG;
  }
  if (!workspace || workspace_bytes < codebook_workspace_bytes(sub_dim, n_samples)) {
    set_error("finetune_codebook: workspace of %zu bytes needed", codebook_workspace_bytes(sub_dim, n_samples));
    return NSN_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 15) {
    set_error("finetune_codebook: the workspace must start on a 16-byte boundary");
    return NSN_ERR_INVALID_ARG;
  }
  const int rc = finetune_run(samples_dev, n_samples, sub_dim, iters, lr, codebook_dev, cos_host, workspace,
                              static_cast<hipStream_t>(stream));
  if (rc == NSN_ERR_HIP) set_error("finetune_codebook: HIP error: %s", hipGetErrorString(hipGetLastError()));
  return rc;
}

int nsn_quantize_codebook(void* codebook_dev, int sub_dim, int n_codes, uint8_t* codes_dev, void* levels_dev,
                          void* stream) {
  if (n_codes != kCodes || (sub_dim != 4 && sub_dim != 8)) {
    set_error("quantize_codebook: unsupported n_codes=%d sub_dim=%d (256 codes of 4 or 8 dims)", n_codes, sub_dim);
    return NSN_ERR_UNSUPPORTED;
  }
  if (!codebook_dev) {
    set_error("quantize_codebook: codebook is NULL");
    return NSN_ERR_INVALID_ARG;
  }
  const int rc = codebook_quantize(codebook_dev, sub_dim, codes_dev, levels_dev, static_cast<hipStream_t>(stream));
  if (rc == NSN_ERR_HIP) set_error("quantize_codebook: HIP error: %s", hipGetErrorString(hipGetLastError()));
  return rc;
}

int nsn_encode(const nsn_shape* shape, const void* codebook_dev, const void* k_fp16, const void* v_fp16,
               int max_new, const int32_t* seq_start_dev, const int32_t* n_new_dev, int batch, int freeze_means,
               const nsn_cache* k_cache, const nsn_cache* v_cache, void* workspace, size_t workspace_bytes,
               void* stream) {
  int rc = check_shape(shape);
  if (rc != NSN_OK) return rc;
  if ((rc = check_cache(shape, k_cache, "K")) != NSN_OK) return rc;
  if ((rc = check_cache(shape, v_cache, "V")) != NSN_OK) return rc;
  if (!codebook_dev || !k_fp16 || !v_fp16 || !seq_start_dev || !n_new_dev || batch < 0 || max_new < 0) {
    set_error("encode: null pointer or negative size");
    return NSN_ERR_INVALID_ARG;
  }
  if (batch == 0 || max_new == 0) return NSN_OK;
  if (!workspace || workspace_bytes < encode_workspace_bytes(*shape, batch, max_new)) {
    set_error("encode: workspace of %zu bytes needed", encode_workspace_bytes(*shape, batch, max_new));
    return NSN_ERR_WORKSPACE;
  }
  rc = encode_launch(*shape, codebook_dev, k_fp16, v_fp16, max_new, seq_start_dev, n_new_dev, batch,
                     freeze_means != 0, *k_cache, *v_cache, workspace, static_cast<hipStream_t>(stream));
  if (rc == NSN_ERR_HIP) set_error("encode: launch failed: %s", hipGetErrorString(hipGetLastError()));
  return rc;
}

static int decode_common(const nsn_shape* shape, const void* codebook_dev, const void* q_fp16,
                         const nsn_cache* k_cache, const nsn_cache* v_cache, const int32_t* seq_lens_dev,
                         int batch, int max_seq_len, const nsn_residual* residual, float softmax_scale,
                         int n_splits, float* out, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != NSN_OK) return rc;
  if ((rc = check_cache(shape, k_cache, "K")) != NSN_OK) return rc;
  if ((rc = check_cache(shape, v_cache, "V")) != NSN_OK) return rc;
  if (!codebook_dev || !q_fp16 || !seq_lens_dev || !out || batch < 0 || n_splits < 0 || max_seq_len < 0 ||
      max_seq_len > shape->max_len) {
    set_error("decode: null pointer, negative size, or max_seq_len=%d beyond max_len=%d", max_seq_len,
              shape->max_len);
    return NSN_ERR_INVALID_ARG;
  }
  if (residual) {
    if (!residual->k_fp16 || !residual->v_fp16 || !residual->lens || residual->capacity < 1 ||
        residual->capacity > 64) {
      set_error("decode: residual needs k, v, lens and a capacity of 1..64 (got %d)", residual->capacity);
      return NSN_ERR_INVALID_ARG;
    }
    if (!decode_use_mfma(*shape)) {
      set_error("decode: the lookup-table kernel (NSN_VARIANT_ALT) has no residual form");
      return NSN_ERR_UNSUPPORTED;
    }
  }
  if ((shape->rope_table || shape->side_bits == 4) && !decode_use_mfma(*shape)) {
    set_error("decode: the lookup-table kernel (NSN_VARIANT_ALT) handles neither rope_table nor side_bits = 4");
    return NSN_ERR_UNSUPPORTED;
  }
  if (batch == 0) return NSN_OK;
  const int splits = decode_pick_splits(*shape, batch, max_seq_len, n_splits);
  if (!workspace || workspace_bytes < decode_workspace_bytes(*shape, batch, splits)) {
    set_error("decode: workspace of %zu bytes needed", decode_workspace_bytes(*shape, batch, splits));
    return NSN_ERR_WORKSPACE;
  }
  rc = decode_launch(*shape, codebook_dev, q_fp16, *k_cache, *v_cache, seq_lens_dev, batch, max_seq_len,
                     softmax_scale, splits, residual, out, workspace, static_cast<hipStream_t>(stream));
  if (rc == NSN_ERR_HIP) set_error("decode: launch failed: %s", hipGetErrorString(hipGetLastError()));
  return rc;
}

int nsn_decode_attention(const nsn_shape* shape, const void* codebook_dev, const void* q_fp16,
                         const nsn_cache* k_cache, const nsn_cache* v_cache, const int32_t* seq_lens_dev,
                         int batch, int max_seq_len, float softmax_scale, int n_splits, float* out,
                         void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(shape, codebook_dev, q_fp16, k_cache, v_cache, seq_lens_dev, batch, max_seq_len, nullptr,
                       softmax_scale, n_splits, out, workspace, workspace_bytes, stream);
}

int nsn_decode_attention_noalloc(const nsn_shape* shape, const void* codebook_dev, const void* q_fp16,
                                 const nsn_cache* k_cache, const nsn_cache* v_cache, const int32_t* seq_lens_dev,
                                 int batch, int max_seq_len, float softmax_scale, int n_splits, float* out,
                                 void* stream) {
  int rc = check_shape(shape);
  if (rc != NSN_OK) return rc;
  if (batch <= 0 || n_splits < 0 || max_seq_len < 0) {
    if (batch == 0) return NSN_OK;
    set_error("decode (noalloc): negative size");
    return NSN_ERR_INVALID_ARG;
  }
  const int splits = decode_pick_splits(*shape, batch, max_seq_len, n_splits);
  const size_t need = decode_workspace_bytes(*shape, batch, splits);
  if (need > kScratchBytes) {
    set_error("decode (noalloc): this call needs %zu scratch bytes, the built-in scratch holds %zu "
              "(batch * n_q_heads * n_splits * 1032 bytes + counters): use nsn_decode_attention with a workspace",
              need, kScratchBytes);
    return NSN_ERR_WORKSPACE;
  }
  void* ptr = scratch_address();
  if (!ptr) return NSN_ERR_HIP;
  const int n_cnt = (int)(decode_counter_bytes(*shape, batch) / sizeof(int));
  scratch_clear_kernel<<<(n_cnt + 255) / 256, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<int*>(ptr), n_cnt);
  if (hipGetLastError() != hipSuccess) {
    set_error("decode (noalloc): launch failed");
    return NSN_ERR_HIP;
  }
  return decode_common(shape, codebook_dev, q_fp16, k_cache, v_cache, seq_lens_dev, batch, max_seq_len, nullptr,
                       softmax_scale, n_splits, out, ptr, kScratchBytes, stream);
}

int nsn_decode_attention_residual(const nsn_shape* shape, const void* codebook_dev, const void* q_fp16,
                                  const nsn_cache* k_cache, const nsn_cache* v_cache,
                                  const int32_t* seq_lens_dev, int batch, int max_seq_len,
                                  const nsn_residual* residual, float softmax_scale, int n_splits, float* out,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!residual) {
    set_error("decode: residual descriptor is null");
    return NSN_ERR_INVALID_ARG;
  }
  return decode_common(shape, codebook_dev, q_fp16, k_cache, v_cache, seq_lens_dev, batch, max_seq_len, residual,
                       softmax_scale, n_splits, out, workspace, workspace_bytes, stream);
}

}  // extern "C"
