/*
 * nsn.h - C ABI of the MI355X (gfx950) coded-KV hot path of NSNQuant (arXiv 2505.18231).
 *
 * Three operations, all executed by hand-written HIP kernels on ONE GPU:
 *   nsn_build_codebook    K-Means codebook on standard-normal samples      (Sec. 3.4)
 *   nsn_encode            Normalize-Shift-Normalize, Hadamard rotation,
 *                         nearest-codeword search, scale adjustment          (Sec. 3.2, 3.3, Eq. 1)
 *   nsn_decode_attention  single-query attention straight from the coded
 *                         cache                                              (App. B)
 * plus nsn_finetune_codebook (Sec. 3.4), nsn_decode_attention_residual (Sec. 3.2 "Residual") and
 * nsn_build_rope_table (keys normalised before the rotary embedding, Sec. 3.2 / App. B).
 *
 * Conventions
 *   - Plain C, no exceptions cross this boundary.  Every call returns an int status:
 *     NSN_OK (0) or a negative NSN_ERR_* code; nsn_last_error() gives a text for the
 *     calling thread's last failure.
 *   - "dev" pointers are device memory owned by the caller (never freed or retained
 *     here); "host" pointers are ordinary host memory.  The library allocates nothing:
 *     scratch comes from a caller workspace sized by nsn_workspace_bytes().
 *   - Kernels are enqueued on the caller's hipStream_t (passed as void*; NULL = the
 *     default stream) and the call returns without synchronising, except
 *     nsn_build_codebook, which returns host results and therefore synchronises.
 *   - No floating-point atomics are used: identical inputs give bit-identical outputs.
 *   - head_dim is 128.  Code formats (sub_dim, n_codes):
 *       (8, 256)    "1-bit": one index byte per 8 rotated channels
 *       (4, 256)    "2-bit": one index byte per 4 rotated channels
 *       (8, 65536)  the paper's own 2-bit format (Sec. 3.4): per 8 rotated channels one index
 *                   byte into a codebook of 256 MAGNITUDE codewords (all entries >= 0; e.g.
 *                   nsn_build_codebook on absolute values of normal samples) plus one sign
 *                   byte (bit i set = channel i negative); 65536 = 256 codewords x 2^8 sign
 *                   patterns.  The codebook passed to the calls still has 256 rows.
 *
 * Coded cache record (one tensor kind, K or V), per (sequence b, kv-head h):
 *   codes  J bytes per token: J = head_dim/sub_dim index bytes; in the sign + index format
 *          J = 32: byte rows j = 0..15 are the indices of sub-vectors 0..15, rows 16..31 their
 *          sign bytes.  Inside one placement unit (see below) the byte of (token t of the
 *          unit, byte row j in [0,J)) sits at the offset that nsn_k_code_offset /
 *          nsn_v_code_offset return:
 *          TILED layout - the (sub_dim, 256) formats without rope_table (either width of side information).
 *          Blocks of 64 tokens, 64 * J bytes each; inside a block one run of J bytes per lane
 *          of the 64-lane wave that reads it; with QS = J / 4 and tb = t % 64:
 *            K:  (t / 64) * 64*J + (16 * (j / QS) + tb % 16) * J + (tb / 16) * QS + j % QS
 *            V:  (t / 64) * 64*J + (16 * (tb % 16 / 4) + 4 * (tb % 4) + j % 4) * J + (tb / 16) * QS + j / 4
 *          K: a lane holds one 32-channel quarter (QS sub-vectors) of tokens tb % 16 = const of
 *          the block's four 16-token tiles, which is its A operand of the 16x16x32 score
 *          contraction; V: a lane holds sub-vectors j % 4 = const of four tokens 16 apart, which
 *          the transposing LDS read turns into "four tokens of one channel" operands.
 *          LEGACY layout - the sign + index format, and every format with rope_table:
 *            K:  t * J + j                                  (token-major)
 *            V:  (t / J) * J*J + j * J + t % J              (blocks of J tokens, sub-vector-major)
 *   norms  one (a, b) fp16 pair per token: b = s1 (first Normalize scale), a = s1*s2*alpha
 *          (second Normalize scale times the scale-adjustment factor of Sec. 3.3).
 *   means  fp16 [n_groups][head_dim]: the Shift vector o of every group of group_size
 *          tokens (group of token t = t / group_size; a single group when group_size = 0),
 *          in the original, un-rotated channel order.
 *   A token dequantises to  b * o_g + a * H^T concat_j C[code_j]   (Sec. 3.2 restore rule).
 *
 * Double quantization (Sec. 3.5; shape->side_bits = 4): the side information is stored in 4 bits,
 * round-to-nearest on the 16 levels  min + step * code  between a group's minimum and maximum
 * (min and step fp16; code = clamp(floor((x - min) / step + 1/2), 0, 15) against the rounded min
 * and step, 0 when step = 0).  norms and means then have these byte layouts instead:
 *   norms  one 164-byte record per 64-token block of a placement unit (record t / 64):
 *            [0,128)   a'_t = fp16(s2 * alpha) of the block's tokens
 *            [128,160) 4-bit codes of s1 (token t & 63 in byte (t & 63) / 2, even token = low nibble)
 *            [160,164) (min, step) fp16 of the block's s1 codes, taken over the tokens the encode
 *                      call wrote; b_t = min + step * code_t and a_t = b_t * a'_t
 *          contiguous: [B][Hkv][max_len / 64] records, paged: [n_pages][Hkv][page_size / 64]
 *   means  one 80-byte record per group, [B][Hkv][NG][80]:
 *            [0,64)    4-bit codes of the 128 channels (channel c in byte c / 2, even = low nibble)
 *            [64,80)   (min, step) fp16 for each of the four 32-channel groups
 *   The first Normalize still divides by fp16(s1); only its stored form is 4-bit.  The Shift
 *   subtracts the DEQUANTISED mean, so the mean's quantisation error is absorbed by the code.
 *   nsn_encode then needs seq_start[b] to be a multiple of 64 (the paper encodes residual-size
 *   chunks), and append mode (freeze_means) re-derives the s1 levels of the block it writes from
 *   the tokens of that call alone.
 *
 * Placement of the units:
 *   contiguous (page_size = 0):
 *       codes [B][Hkv][max_len * J] bytes, norms [B][Hkv][max_len] pairs
 *   paged (page_size > 0, a multiple of 64):
 *       codes [n_pages][Hkv][page_size * J], norms [n_pages][Hkv][page_size],
 *       block_table dev int32 [B][max_len / page_size]: physical page of each logical page
 *   means are never paged: fp16 [B][Hkv][NG][head_dim], NG = nsn_max_groups(shape).
 */
#ifndef NSN_H
#define NSN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  NSN_OK = 0,
  NSN_ERR_INVALID_ARG = -1, /* null pointer, negative size, misaligned start, ... */
  NSN_ERR_UNSUPPORTED = -2, /* head_dim != 128, a (sub_dim, n_codes) pair not listed above, ... */
  NSN_ERR_WORKSPACE = -3,   /* workspace missing or smaller than nsn_workspace_bytes() */
  NSN_ERR_HIP = -4          /* a HIP runtime call or kernel launch failed */
};

enum { NSN_OP_ENCODE = 0, NSN_OP_DECODE = 1, NSN_OP_CODEBOOK = 2 };

typedef struct nsn_shape {
  int32_t head_dim;   /* 128 */
  int32_t sub_dim;    /* 8 or 4 */
  int32_t n_codes;    /* 256, or 65536 with sub_dim 8: the sign + index format (see above) */
  int32_t n_q_heads;  /* multiple of n_kv_heads; n_q_heads / n_kv_heads <= 8 (the decode kernel
                         takes four query heads per kv head per launch: five to eight heads run
                         as two launches, the second reading the cache again) */
  int32_t n_kv_heads;
  int32_t group_size; /* G: tokens sharing one Shift mean; multiple of 64 (the paper uses 64),
                         or 0 = one group per sequence */
  int32_t page_size;  /* 0 = contiguous; else tokens per page, multiple of 64 */
  int32_t max_len;    /* token capacity per sequence, multiple of 64 (and of page_size) */
  const void* rope_table; /* NULL: keys are coded as given.  Else dev table written by
                             nsn_build_rope_table for a max_len >= this one: the K input of
                             nsn_encode holds keys BEFORE the rotary embedding (Sec. 3.2 "NSN applied
                             to key and value"); see nsn_build_rope_table for what changes */
  int32_t side_bits;      /* 0 or 16: fp16 norms and means; 4: double quantization (see above) */
} nsn_shape;

typedef struct nsn_cache {
  uint8_t* codes;             /* dev */
  void* norms;                /* dev, fp16 pairs (a, b) */
  void* means;                /* dev, fp16 */
  const int32_t* block_table; /* dev, paged layout only (else NULL) */
} nsn_cache;

/*
 * The residual of Sec. 3.2: the most recent tokens of every sequence, kept in fp16 until a
 * whole group of them is encoded at once.  Rows [0, lens[b]) of a sequence are its tokens
 * at positions seq_lens[b] .. seq_lens[b] + lens[b] - 1 (oldest first); the caller owns the
 * buffers, appends to them and empties them (by passing them to nsn_encode and resetting
 * lens) when they are full.
 */
typedef struct nsn_residual {
  const void* k_fp16;  /* dev fp16 [batch][n_kv_heads][capacity][head_dim] */
  const void* v_fp16;  /* dev fp16, same shape */
  const int32_t* lens; /* dev int32 [batch], 0 .. capacity */
  int32_t capacity;    /* rows per (sequence, kv head): 1 .. 64 (the paper uses 64) */
} nsn_residual;

/*
 * Keys normalised before the rotary embedding (Sec. 3.2 "NSN applied to key and value", App. B).
 * The embedding meant is the Llama-family one: channel i and channel i + 64 form a pair that
 * turns by the angle position * inv_freq[i]; the position of a token is its index in the sequence.
 * With shape->rope_table set,
 *   nsn_encode  runs Normalize-Shift-Normalize on the K rows as given (before the embedding),
 *               turns v_nsn of every token by its position, then rotates, searches and adjusts as
 *               usual; b and the stored mean o are those of the un-embedded keys.  V is unaffected.
 *   nsn_decode_attention[_residual]  take the query AFTER the embedding and turn the mean inside
 *               the kernel:  score_t = softmax_scale * (a_t HT(q) . C[codes_t] + b_t q . RoPE_t(o_g(t))).
 *               Residual K rows are the keys after the embedding (as attention uses them); the
 *               caller keeps the un-embedded copies for the nsn_encode call that empties the residual.
 * The table holds cosines and sines evaluated in fp64: of 64 * block * inv_freq[i] per 64-token
 * block (fp64 and fp32 copies), of j * inv_freq[i] for j < 64 (fp64, and as fp16 hi + lo pairs for
 * the matrix cores); angles of a token are composed from the two by the addition theorems.  A table
 * built for a larger max_len serves every smaller one.
 *   inv_freq_host  host fp32 [64]
 *   max_len        positions covered, a positive multiple of 64
 *   table_dev      out, dev, nsn_rope_table_bytes(max_len) bytes, 256-byte aligned
 * Enqueues one kernel on `stream`; the table may be used by later calls on the same stream.
 * Errors: INVALID_ARG (null pointer, max_len, table_bytes too small), HIP.
 */
size_t nsn_rope_table_bytes(int max_len);
int nsn_build_rope_table(const float* inv_freq_host, int max_len, void* table_dev, size_t table_bytes,
                         void* stream);

/* Byte offset of code byte row j of token t inside a placement unit of a cache of this shape
 * (see "codes" above); -1 for an invalid shape, t < 0 or j outside [0, J). */
int64_t nsn_k_code_offset(const nsn_shape* shape, int64_t t, int j);
int64_t nsn_v_code_offset(const nsn_shape* shape, int64_t t, int j);
/* Number of mean vectors kept per (sequence, kv-head): max_len / group_size rounded up, or 1. */
int nsn_max_groups(const nsn_shape* shape);
/* Text of the calling thread's most recent error ("" if none). Never NULL. */
const char* nsn_last_error(void);

/* Kernel variants.  Each operation has a default kernel and one alternative that computes the same
 * result another way; the alternative exists for cross-checks and measurements.
 *   NSN_OP_ENCODE  NSN_VARIANT_DEFAULT  nearest-codeword distances (Eq. 1) contracted on the matrix cores
 *                  NSN_VARIANT_ALT      the same distances by an fp32 vector scan (index-only and
 *                                       sign + index formats without rope_table)
 *   NSN_OP_DECODE  NSN_VARIANT_DEFAULT  matrix-core attention kernels (every format)
 *                  NSN_VARIANT_ALT      App. B as written: a query x codebook score table, fp32 throughout
 *                                       (index-only formats with fp16 side information, no rope_table, no
 *                                       residual; other calls fail with NSN_ERR_UNSUPPORTED)
 * The choice is process-wide and applies to calls made after this one returns.  Its initial value is
 * taken from the environment, once, at the library's first use: NSN_ENCODE_IMPL=valu and
 * NSN_DECODE_IMPL=lut select the alternatives.  Returns the previous variant, or NSN_ERR_INVALID_ARG. */
enum { NSN_VARIANT_DEFAULT = 0, NSN_VARIANT_ALT = 1 };
int nsn_select_variant(int op, int variant);

/*
 * Workspace (device bytes) an operation needs.
 *   NSN_OP_ENCODE   : n = max_new (token stride of the inputs), n_splits ignored
 *   NSN_OP_DECODE   : n ignored, n_splits as passed to nsn_decode_attention (0 = auto).
 *                     The decode workspace starts with arrival counters: fill it with zeros
 *                     ONCE after allocating it; every call leaves it ready for the next one.
 *                     Calls that share one workspace must not overlap in time.
 *   NSN_OP_CODEBOOK : n = n_samples, batch and n_splits ignored; the workspace starts on a
 *                     16-byte boundary (INVALID_ARG otherwise)
 * Returns 0 for an invalid shape.
 */
size_t nsn_workspace_bytes(const nsn_shape* shape, int op, int batch, int64_t n, int n_splits);

/*
 * K-Means codebook on standard-normal data (Sec. 3.4, the K-Means baseline; the fine-tuning
 * step is nsn_finetune_codebook).
 *   samples_dev   dev fp32 [n_samples][sub_dim], drawn by the caller (the library holds no
 *                 random generator); the first n_codes samples are the initial centroids
 *   iters         Lloyd iterations: assign to the nearest centroid in squared Euclidean
 *                 distance (lowest index on ties, decided in fp64), then replace every
 *                 non-empty cluster's centroid by its fp64 mean
 *   codebook_dev  out, dev fp16 [n_codes][sub_dim]: final centroids rounded to fp16 once
 *   mse_host      out, host double[1]: mean squared error per dimension of the samples
 *                 against the rounded codebook (may be NULL)
 * Synchronises the stream before returning.  Errors: INVALID_ARG (null pointers,
 * n_samples < n_codes, iters < 0), UNSUPPORTED (sub_dim, n_codes), WORKSPACE, HIP.
 */
int nsn_build_codebook(const float* samples_dev, int64_t n_samples, int sub_dim, int n_codes,
                       int iters, void* codebook_dev, double* mse_host, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * Fine-tune a codebook for cosine distance on standard-normal data (Sec. 3.4): `iters` times,
 * assign every sample to its nearest codeword (Eq. 1, as nsn_build_codebook does) and take one
 * full-batch gradient step of  mean_x (1 - cos(x, C[k(x)]))  with the assignment held fixed
 * (the lookup is not differentiated):
 *     C[k] += lr / (N |C[k]|) * (S_k - (S_k . c^) c^),   S_k = sum of x / |x| over the samples of k,
 *     c^ = C[k] / |C[k]|.   Zero samples and zero codewords are left out.
 * The paper names neither optimiser nor rate nor step count; plain gradient steps with the
 * caller's `lr` are this library's reading.
 *   samples_dev   dev fp32 [n_samples][sub_dim]
 *   codebook_dev  in/out, dev fp16 [n_codes][sub_dim]: the start (e.g. from nsn_build_codebook);
 *                 steps run in fp64, the result is rounded to fp16 once
 *   cos_host      out, host double[2]: mean cosine similarity between the samples and their
 *                 quantised versions before and after (may be NULL)
 *   workspace     nsn_workspace_bytes(shape, NSN_OP_CODEBOOK, 0, n_samples, 0) bytes
 * Synchronises the stream before returning.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.
 */
int nsn_finetune_codebook(const float* samples_dev, int64_t n_samples, int sub_dim, int n_codes,
                          int iters, double lr, void* codebook_dev, double* cos_host,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Codebook entries on 16 levels (Sec. 3.5, "we also apply 4-bit quantization to codebook entries"):
 * every entry is replaced by fp16(min + step * code), code = the 4-bit round-to-nearest level of
 * the entry between the smallest and the largest entry of the whole codebook (one fp16 (min, step)
 * pair per codebook: the paper does not state a grouping).  The kernels keep reading an fp16
 * codebook; the 4-bit form matters for where a codebook is stored, not for these kernels, whose
 * LDS table is an expanded, replicated copy anyway.
 *   codebook_dev  in/out, dev fp16 [n_codes][sub_dim]
 *   codes_dev     out, dev u8 [n_codes * sub_dim] (one code per byte), may be NULL
 *   levels_dev    out, dev fp16 [2] = (min, step), may be NULL
 * One kernel on `stream`, no synchronisation.  Errors: INVALID_ARG, UNSUPPORTED (sub_dim, n_codes), HIP.
 */
int nsn_quantize_codebook(void* codebook_dev, int sub_dim, int n_codes, uint8_t* codes_dev,
                          void* levels_dev, void* stream);

/*
 * Encoder (Sec. 3.2 steps 1-3, Hadamard rotation of Sec. 2, Eq. 1 on contiguous sub-vectors
 * of the rotated token, scale adjustment of Sec. 3.3).  For every sequence b it encodes the
 * n_new[b] tokens found in k_fp16 / v_fp16 and writes them at cache positions
 * [seq_start[b], seq_start[b] + n_new[b]).
 *   codebook_dev  dev fp16 [256][sub_dim]
 *   k_fp16,v_fp16 dev fp16 [batch][n_kv_heads][max_new][head_dim]; rows >= n_new[b] are ignored
 *   seq_start,n_new dev int32 [batch]
 *   freeze_means  0: the Shift mean of every group touched is computed from the new tokens
 *                    (seq_start[b] must then be a multiple of group_size, or 0 when
 *                    group_size = 0) and stored;
 *                 1: append mode - the stored mean of the token's group is used unchanged,
 *                    so a new token never forms a one-token group (the group must exist).
 *   Storage rounding: b, o and a are rounded to fp16 (nearest even, one rounding from fp64);
 *   the rounded b and o are the values used in the later steps.
 *   A zero scale (s1 = 0 or s2 = 0) stores a zero vector and a zero scale; the adjustment
 *   factor is 1 when (rotated token) . (its quantised version) <= 1e-12 * head_dim.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.  Out-of-range positions
 * (seq_start + n_new > max_len) are clipped on the device: such tokens are not written.
 */
int nsn_encode(const nsn_shape* shape, const void* codebook_dev, const void* k_fp16,
               const void* v_fp16, int max_new, const int32_t* seq_start_dev,
               const int32_t* n_new_dev, int batch, int freeze_means, const nsn_cache* k_cache,
               const nsn_cache* v_cache, void* workspace, size_t workspace_bytes, void* stream);

/*
 * One decode step of attention over the coded cache (App. B; the mean enters as stored unless
 * shape->rope_table is set, see nsn_build_rope_table):
 *   score_t = softmax_scale * ( a^k_t * HT(q) . C[codes^k_t] + b^k_t * q . o^k_g(t) )
 *   out     = sum_t softmax(score)_t * ( a^v_t * H^T C[codes^v_t] + b^v_t * o^v_g(t) )
 *   q_fp16       dev fp16 [batch][n_q_heads][head_dim]; query head hq reads kv head
 *                hq / (n_q_heads / n_kv_heads)
 *   seq_lens_dev dev int32 [batch], cached tokens per sequence (0 gives a zero output row)
 *   max_seq_len  host upper bound of seq_lens (sizes the launch; <= shape->max_len)
 *   n_splits     partitions of the token axis processed by separate workgroups and merged
 *                with fp32 running max / sum (0 = choose from the shape)
 *   out          dev fp32 [batch][n_q_heads][head_dim]
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.
 */
int nsn_decode_attention(const nsn_shape* shape, const void* codebook_dev, const void* q_fp16,
                         const nsn_cache* k_cache, const nsn_cache* v_cache,
                         const int32_t* seq_lens_dev, int batch, int max_seq_len,
                         float softmax_scale, int n_splits, float* out, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * The same decode step with the fp16 residual of Sec. 3.2 taking part in the softmax:
 *   out = softmax(softmax_scale * q [K_coded ; K_residual]^T) [V_coded ; V_residual]
 * where the coded part is exactly nsn_decode_attention's and the residual rows enter with
 * their fp16 values (fp32 accumulation).  seq_lens_dev counts coded tokens only; a sequence
 * with no coded and no residual token gives a zero output row.  All other arguments, the
 * workspace and its rules are those of nsn_decode_attention.
 * Errors: INVALID_ARG (also capacity outside 1..64), UNSUPPORTED, WORKSPACE, HIP.
 */
int nsn_decode_attention_residual(const nsn_shape* shape, const void* codebook_dev,
                                  const void* q_fp16, const nsn_cache* k_cache,
                                  const nsn_cache* v_cache, const int32_t* seq_lens_dev,
                                  int batch, int max_seq_len, const nsn_residual* residual,
                                  float softmax_scale, int n_splits, float* out, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * nsn_decode_attention for callers that cannot allocate or hand over device memory for scratch
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * operation and arguments, without a workspace.  The arrival counters and split partials live in a
 * fixed 4 MiB array inside the library's device image (one copy per GPU, held until the process
 * ends); the call allocates nothing and clears the counters it uses with a small kernel on `stream`.
 *   - Needs batch * n_q_heads * n_splits * 1032 bytes + 256 bytes per (sequence, query head), rounded up
 *     to 256: calls that need more than 4 MiB fail with NSN_ERR_WORKSPACE (use nsn_decode_attention).
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU (different streams,
 *     different host threads) race; calls on one stream do not.
 * Errors: as nsn_decode_attention, plus NSN_ERR_HIP if the array's address cannot be obtained.
 */
int nsn_decode_attention_noalloc(const nsn_shape* shape, const void* codebook_dev, const void* q_fp16,
                                 const nsn_cache* k_cache, const nsn_cache* v_cache,
                                 const int32_t* seq_lens_dev, int batch, int max_seq_len,
                                 float softmax_scale, int n_splits, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NSN_H */
