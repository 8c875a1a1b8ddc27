// Decode attention over the coded cache (App. B) for the tiled code layout: the gfx950 kernel.
//
// Arithmetic (per query head): score_t = scale (a^k_t HT(q) . C[codes^k_t] + b^k_t q . o^k_g),
// p = softmax(score), out = H^T sum_t p_t a^v_t C[codes^v_t] + sum_g (sum_{t in g} p_t b^v_t) o^v_g.
//
// How the 64 tokens of a group map onto a wave (lane = 16 c + n, c = 0..3, n = 0..15):
//   * scores: v_mfma_f32_16x16x32_f16 with the gathered KEY CODEWORDS as the A operand (row = token
//     16 tile + n of the group, the lane's eight k-slots = the eight channels it gathered: lane group c
//     owns channels [32 c, 32 c + 32)) and the rotated query as the B operand.  The sixteen columns carry
//     four heads x (fp16 hi part, fp16 lo part) x two tiles: tile parity p uses columns [4p, 4p+4) for hi
//     and [8+4p, 12+4p) for lo, all other columns of that B operand are zero, so two tiles accumulate
//     into one result and four k-steps x four tiles = sixteen matrix instructions give a group's scores
//     with ~22 significant bits of the query.  Adding column n and column n ^ 8 leaves, in lane
//     (rho = lane / 16, n): tile n / 4, head n % 4, tokens 16 tile + 4 rho + {0,1,2,3}.
//   * softmax per lane (one head, four tokens), running max kept lazily (rescale only when a score
//     exceeds it by 2^5), in log2 units.
//   * values: that register IS the A operand of v_mfma_f32_4x4x4_16B_f16 (block = lane / 4 holds four
//     tokens of one head row each), no transpose.  The B operand must hold four TOKENS of one channel
//     per lane, while a gathered codeword is four channels of one token: ds_read_b64_tr_b16 transposes
//     the gather on its way out of LDS (within 16 lanes, result lane 4 m + e, slot k <- source lane
//     4 k + m, element e).  With cbsz = 2 the four blocks of a 16-lane group share the weights of block
//     `abid` (= tile), each taking another sub-vector: 32 gathers + 32 matrix instructions per group, and
//     the accumulators are out_rot[head][channel] partial sums per 16-lane group.
//   * the fp16 weights are p a^v / A with A a power of two >= every a^v seen so far (rescaled lazily like
//     the running max), so the value contraction does not depend on the scale of V.
// One workgroup per (split, kv head, sequence) - or, for batches of 128 units and more, one persistent
// workgroup per compute unit that takes an equal run of all groups (see the kernel's FLAT flag) - 8 waves,
// one 64 KiB codebook table replicated per LDS bank group (conflict-free gathers: one v_perm_b32 forms the
// address from a code byte).  Cache bytes are fetched two groups ahead into rotating register sets.  The fp16 residual (Sec. 3.2) is one more
// group whose four 16-token tiles are taken by waves 0..3 of the last split before their own groups (a
// quarter group each: a ninth wave would cap every wave at 168 registers, and a whole extra group on one
// wave would lengthen a four-group loop by a quarter).  Waves merge through LDS once; splits
// merge through fp32 partials in the workspace, the last wave to arrive (integer counter per query
// head) finishing the head: merge, one inverse Hadamard in registers, mean-vector term, output.
#include <algorithm>
#include <type_traits>

#include "nsn_host.h"

namespace nsn {
namespace tile {

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2v __attribute__((ext_vector_type(2)));
typedef short s4v __attribute__((ext_vector_type(4)));
typedef uint32_t u2v __attribute__((ext_vector_type(2)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));

constexpr int kPartialStride = 2 * kHeadDim + 2;  // rotated acc, mean-term acc, m (log2 units), l
constexpr float kLazyMaxLog2 = 5.0f;              // rescale only when a score beats the running max by 2^5
constexpr float kWeightScale = 1024.0f;           // fp16 weights carry 2^10 / A: small weights stay normal numbers
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
// (code byte k of `codes`) << 8 | lane offset: the LDS address of a table entry (the table starts at 0)
template <int K>
__device__ __forceinline__ uint32_t table_addr(uint32_t codes, uint32_t laneoff) {
  return perm_b32(codes, laneoff, 0x0c0c0400u + (K << 8));
}

#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ u2v lds_read64(uint32_t addr) { return *(const u2v __attribute__((address_space(3)))*)(addr); }
__device__ __forceinline__ u4v lds_read128(uint32_t addr) { return *(const u4v __attribute__((address_space(3)))*)(addr); }
__device__ __forceinline__ float lds_read32f(uint32_t addr) { return *(const float __attribute__((address_space(3)))*)(addr); }
__device__ __forceinline__ h4 lds_tr64(uint32_t addr) {
  return __builtin_bit_cast(h4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4v __attribute__((address_space(3)))*)(addr)));
}
__device__ __forceinline__ void lds_write128(uint32_t addr, u4v v) { *(u4v __attribute__((address_space(3)))*)(addr) = v; }
__device__ __forceinline__ void lds_write64(uint32_t addr, u2v v) { *(u2v __attribute__((address_space(3)))*)(addr) = v; }
__device__ __forceinline__ void lds_write32(uint32_t addr, uint32_t v) { *(uint32_t __attribute__((address_space(3)))*)(addr) = v; }
#else
__device__ __forceinline__ u2v lds_read64(uint32_t) { return u2v{0, 0}; }
__device__ __forceinline__ u4v lds_read128(uint32_t) { return u4v{0, 0, 0, 0}; }
__device__ __forceinline__ float lds_read32f(uint32_t) { return 0.f; }
__device__ __forceinline__ h4 lds_tr64(uint32_t) { return h4{}; }
__device__ __forceinline__ void lds_write128(uint32_t, u4v) {}
__device__ __forceinline__ void lds_write64(uint32_t, u2v) {}
__device__ __forceinline__ void lds_write32(uint32_t, uint32_t) {}
#endif

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// v_permlane16_swap / v_permlane32_swap exchange the odd 16-lane rows of `a` with the even rows of `b`
// (the upper half of `a` with the lower half of `b`).  Written as instructions: the compiler's two-result
// builtins for them were seen to return the first result twice.  The instruction reads other lanes'
// registers, which needs two idle cycles after a vector instruction wrote them (s_nop 1).
__device__ __forceinline__ void lane_swap16(float& a, float& b) {
  asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void lane_swap32(float& a, float& b) {
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
// value of lane (lane ^ 16) / (lane ^ 32): a swap of two copies (no LDS traffic)
__device__ __forceinline__ float xor16(float v) {
  float a = v, b = v;
  lane_swap16(a, b);  // a: rows (0,0,2,2), b: rows (1,1,3,3)
  return ((threadIdx.x >> 4) & 1) ? a : b;
}
__device__ __forceinline__ float xor32(float v) {
  float a = v, b = v;
  lane_swap32(a, b);  // a: the lower half twice, b: the upper half twice
  return ((threadIdx.x >> 5) & 1) ? a : b;
}
// value of lane (lane ^ M): DPP inside a 16-lane row, register swaps across rows
template <int M>
__device__ __forceinline__ float xor_reg(float v) {
  if constexpr (M == 16)
    return xor16(v);
  else if constexpr (M == 32)
    return xor32(v);
  else
    return xor_lane<M>(v);
}
// max of finite or infinite values (never NaN here): the plain instruction, without the operand
// canonicalisation that fmaxf() adds under IEEE rules (one extra instruction per operand)
__device__ __forceinline__ float max3f(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float max2f(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// reductions over the sixteen lanes that share (lane % 4), i.e. one query head
__device__ __forceinline__ float head_max(float v) {
  v = max2f(v, dpp_mov<0x124>(v));  // row_ror:4
  v = max2f(v, dpp_mov<0x128>(v));  // row_ror:8
  v = max2f(v, xor16(v));
  v = max2f(v, xor32(v));
  return v;
}
__device__ __forceinline__ float head_sum(float v) {
  v += dpp_mov<0x124>(v);
  v += dpp_mov<0x128>(v);
  v += xor16(v);
  v += xor32(v);
  return v;
}
__device__ __forceinline__ float wave_max_all(float v) {
  v = max2f(v, dpp_mov<0xB1>(v));  // quad_perm [1,0,3,2]
  v = max2f(v, dpp_mov<0x4E>(v));  // quad_perm [2,3,0,1]
  return head_max(v);
}
__device__ __forceinline__ float wave_sum_all(float v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  return head_sum(v);
}
// value held by lane j of the caller's quad
template <int J>
__device__ __forceinline__ float quad_bcast(float v) {
  return dpp_mov<J | (J << 2) | (J << 4) | (J << 6)>(v);
}

__device__ __forceinline__ float half_lo_f(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu)); }
__device__ __forceinline__ float half_hi_f(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); }
__device__ __forceinline__ void st_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// LDS plan (dynamic block, starts at LDS address 0 because the gathers form absolute addresses):
//   [0, 64 KiB)   codebook table: entry (code c, copy p) at c * 256 + p * (2 * SUB): 32 copies of 8 bytes
//                 (SUB = 4) or 16 copies of 16 bytes (SUB = 8)
//   query block   fp16 hi / lo of the rotated, pre-scaled query [4][128] each; the same of the unrotated
//                 query (residual tiles); 128 zero bytes; q . o^k of the split's first Shift group (four
//                 heads); the unrotated query in fp32 [4][128]
//   merge block   per wave: rotated-domain sums [4][128] fp32, mean-term sums [4][128] fp32, (m, l) x 4
//   residual rows per wave 0..3: 16 fp16 key rows at a stride of 272 bytes, 16 value rows at 264
//                 (residual launches only)
template <int NW>
struct Smem {
  static constexpr int kQhi = kTableBytes, kQlo = kQhi + 1024, kUhi = kQlo + 1024, kUlo = kUhi + 1024;
  static constexpr int kZero = kUlo + 1024, kQoFirst = kZero + 128, kQorig = kZero + 256;
  static constexpr int kMerge = kQorig + 2048;
  static constexpr int kMergeWave = 2048 + 2048 + 256;
  static constexpr int kBytes = kMerge + NW * kMergeWave;
  // residual launches: 16 key rows (stride 272 bytes) and 16 value rows (stride 264) for each of four waves
  static constexpr int kResKStride = 272, kResVStride = 264;
  static constexpr int kResWave = 16 * kResKStride + 16 * kResVStride;
  static constexpr int kRes = kBytes;
  static constexpr int kBytesRes = kRes + 4 * kResWave;
  static_assert(kBytesRes <= 160 * 1024, "LDS of one compute unit");
};

// one 64-token group's cache bytes as a lane needs them
template <int CW>
struct GroupRegs {
  uint32_t kc[CW], vc[CW];  // the lane's code bytes of the group (tiled layout: CW dwords per tensor)
  uint4 nk, nv;             // (a, b) fp16 pairs of the lane's four tokens 16 tile + 4 rho + {0..3}
  uint32_t ok, ov;          // channels 2 lane, 2 lane + 1 of the group's Shift vectors (fp16 pairs)
  // 4-bit side information (DQ): nk / nv = {a' of the four tokens (two words), their four s1 nibbles, the
  // block's (min, step)}; ok / ov = the byte with the two channels' nibbles, okp / ovp = (min, step) of the
  // lane's 32-channel group
  uint32_t okp, ovp;
};
// min + step * code of a 4-bit level (par = fp16 pair (min, step))
__device__ __forceinline__ float dq_level(uint32_t par, uint32_t code) {
  return fmaf(half_hi_f(par), (float)code, half_lo_f(par));
}

// POW2: group_size (if any) and, for paged caches, page_size are powers of two: group and page indices are
// shifts (the other instance divides: about 35 scalar instructions per index)
// PAGED: the caches are paged (block tables); the other instance never reads a block table and can
// fetch its first group before the sequence length is known
// FLAT: the launch is one persistent workgroup per compute unit.  All 64-token groups of all (sequence,
// kv head) units form one list (unit by unit, a unit without coded tokens counts as one group); workgroup c
// takes the c-th of n_splits equal runs of that list, which is a sequence of segments: (unit, first group,
// number of groups).  A unit that is cut by a run boundary is merged through partial results exactly as a
// split one is in the other instance.  Ragged batches and batches with more units than compute units keep
// every compute unit busy this way, and the codebook table is built once per workgroup.
// Every unit takes kSegCost list slots in front of its groups: a segment costs about as much as that many
// groups (query rotation, two barriers, the merge of the waves, a cold start of the loads), so that runs with
// many short units get fewer groups.  A run that ends inside those slots leaves the unit to the next run.
constexpr int kSegCost = 32;
// DQ: norms and means are stored in 4 bits (Sec. 3.5): 164-byte norm records per 64-token block, 80-byte mean records
template <int SUB, int NW, bool POW2, bool PAGED, bool FLAT, bool DQ>
__global__ __launch_bounds__(NW * 64) void dec_tile_kernel(Geometry g, const __half* __restrict__ codebook,
                                                           const __half* __restrict__ q, CacheView kc, CacheView vc,
                                                           const int32_t* __restrict__ seq_lens, int batch,
                                                           float scale_log2e, int n_splits, int per, float* partial,
                                                           int* counters, ResidualView res, int head_off, int r_pass,
                                                           float* __restrict__ out) {
  static_assert(NW == 8, "prologue work split: 512 threads fill the table, waves 0..3 rotate the query");
  constexpr int NSV = kHeadDim / SUB;  // sub-vectors (= code bytes) per token
  constexpr int CW = NSV / 4;          // code dwords per lane, group and tensor
  using SM = Smem<NW>;
  using Regs = GroupRegs<CW>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

  const int r = r_pass;
  const int tid = threadIdx.x, lane0 = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cap_tokens = g.page_tokens * g.pages_per_seq;
  // the segment at hand (!FLAT: the launch's one (split, kv head, sequence))
  int split = FLAT ? 0 : blockIdx.x, h = FLAT ? 0 : blockIdx.y, b = FLAT ? 0 : blockIdx.z;
  int t0 = split * per;
  int64_t mean_base = (int64_t)(b * g.n_kv_heads + h) * g.n_groups_max;

  // ---- loads that do not depend on the sequence length go out first ------------------------------
  // (all unconditional, so that the wait for the codebook can leave the later ones in flight)
  typedef typename std::conditional<SUB == 4, uint2, uint4>::type cw_t;
  const cw_t cw_reg = reinterpret_cast<const cw_t*>(codebook)[tid >> 1];  // two threads per code row

  // ---- FLAT: this workgroup's run of the group list (every wave computes the same numbers) --------
  const int hkv = g.n_kv_heads;
  int run_q = 0, run_pos = 0, run_end = 0, seg_g = 0;  // run length, list position, end of the run, slot inside the unit
  // codebook table: thread (code = tid / 2, half = tid % 2) fills eight 16-byte slots of its half row, starting
  // at a slot that depends on the code so that the 64 stores of a wave spread over all banks
  auto fill_table = [&]() {
    const int code = tid >> 1, half = tid & 1;
    u4v v;
    if constexpr (SUB == 4)
      v = u4v{cw_reg.x, cw_reg.y, cw_reg.x, cw_reg.y};
    else
      v = u4v{cw_reg.x, cw_reg.y, cw_reg.z, cw_reg.w};
    const uint32_t row = code * 256 + half * 128;
#pragma unroll
    for (int u = 0; u < 8; ++u) lds_write128(row + (((u + code) & 7) << 4), v);
  };
  if constexpr (FLAT) {
    auto groups_of = [](int len) { return max(1, (len + 63) >> 6); };
    // list positions taken by the sequences of one 64-sequence block: this lane's sequence, and the inclusive
    // prefix sums over the lanes
    auto block_sizes = [&](int b0, int& n, int& incl) {
      n = (b0 + lane0 < batch) ? (groups_of(seq_lens[b0 + lane0]) + kSegCost) * hkv : 0;
      incl = n;
      static_for<6>([&](auto kc_) {
        constexpr int d = 1 << decltype(kc_)::value;
        const int up = __shfl_up(incl, d);
        incl += (lane0 >= d) ? up : 0;
      });
    };
    int n0, incl0;
    block_sizes(0, n0, incl0);  // (the table is filled while these lengths are on their way)
    fill_table();
    int total = __builtin_amdgcn_readlane(incl0, 63);
    for (int b0 = 64; b0 < batch; b0 += 64) {
      int n, incl;
      block_sizes(b0, n, incl);
      total += __builtin_amdgcn_readlane(incl, 63);
    }
    run_q = (total + n_splits - 1) / n_splits;
    run_pos = (int)blockIdx.x * run_q;
    if (run_pos >= total) return;  // (all waves alike, before any barrier)
    run_end = min(total, run_pos + run_q);
    // the sequence that holds list position run_pos: sequences are laid out one after the other, each as
    // n_kv_heads units of its group count
    int before = 0;  // list positions in front of the 64-sequence block at hand
    for (int b0 = 0; b0 < batch; b0 += 64) {
      int n = n0, incl = incl0;
      if (b0 > 0) block_sizes(b0, n, incl);
      const int n_before = __popcll(__ballot(b0 + lane0 < batch && before + incl <= run_pos));  // sequences that end at or before it
      const int n_here = min(64, batch - b0);
      if (n_before < n_here) {
        b = b0 + n_before;
        const int incl_b = __builtin_amdgcn_readlane(incl, n_before), n_b = __builtin_amdgcn_readlane(n, n_before);
        const int off = run_pos - (before + incl_b - n_b);  // position inside the sequence's n_kv_heads units
        const int slots = n_b / hkv;
        h = off / slots;
        seg_g = off - h * slots;  // (position among the unit's slots)
        break;
      }
      before += __builtin_amdgcn_readlane(incl, 63);
    }
  }

  bool first_segment = true;
  // FLAT: the next segment's sequence length, query row and first mean row are fetched a segment ahead
  int len_cur = 0, nb = 0, nh = 0;
  __half2 q2_next = __half2{};
  uint32_t okf_next = 0u, okfp_next = 0u;
  // PAGED: the wave's window of block-table entries (see load_window); the first group of a pass loads it
  int win0 = -(1 << 30), win_k = 0, win_v = 0, nwin_k = 0, nwin_v = 0;
  if constexpr (FLAT) len_cur = seq_lens[b];
  for (;;) {  // FLAT: one pass per segment of the run; otherwise a single pass
  // Everything a pass derives from the lane number is derived anew in each pass: values that the compiler
  // could compute once in front of the segment loop would stay in registers through all of it, and this
  // kernel has none to spare.
  int lane = lane0;
  if constexpr (FLAT) asm volatile("" : "+v"(lane));
  const int rho = lane >> 4, n16 = lane & 15, head = lane & 3, tile_of_lane = n16 >> 2;
  // ---- loads of one group (all unconditional: callers clamp the group index into the cache) ----
  const uint32_t lane_code_off = lane * NSV;
  const uint32_t norm_off = (16 * tile_of_lane + 4 * rho) * 4;  // bytes: the lane's first token of the group
  const uint32_t lane_x4 = lane * 4;
  // Paged caches: the wave keeps 64 consecutive block-table entries of its sequence in two registers (lane i:
  // page win0 + i, clamped into the sequence's table row) and picks a group's entries with lane reads.  An
  // entry loaded right before its use would make the wave wait for every load it has in flight (loads return
  // in order); the window is loaded once per segment (the persistent instance asks for the next segment's
  // window when it leaves its main loop) and again only when a group lies beyond it.
  auto load_window = [&](int bb, int w0, int& wk, int& wv) {
    const int64_t e = (int64_t)bb * g.pages_per_seq + min(w0 + lane, g.pages_per_seq - 1);
    wk = kc.block_table[e], wv = vc.block_table[e];
  };
  // token index (counted over the whole buffer) of the first token of the group that starts at token tg
  auto group_bases = [&](int tg, int64_t& kbase, int64_t& vbase) {
    if constexpr (!PAGED) {
      kbase = vbase = (int64_t)(b * g.n_kv_heads + h) * g.page_tokens + tg;
    } else {
      const int page = POW2 ? tg >> g.page_shift : tg / g.page_tokens;
      const int tin = POW2 ? tg & (g.page_tokens - 1) : tg % g.page_tokens;
      if ((unsigned)(page - win0) >= 64u) {  // wave-uniform
        win0 = page & ~63;
        load_window(b, win0, win_k, win_v);
      }
      const int pk = __builtin_amdgcn_readlane(win_k, page - win0), pv = __builtin_amdgcn_readlane(win_v, page - win0);
      kbase = ((int64_t)pk * g.n_kv_heads + h) * g.page_tokens + tin;
      vbase = ((int64_t)pv * g.n_kv_heads + h) * g.page_tokens + tin;
    }
  };
  auto shift_group = [&](int tg) -> int {
    return g.group_size <= 0 ? 0 : POW2 ? tg >> g.group_shift : tg / g.group_size;
  };
  // tg: first token of the group (a multiple of 64 inside the cache).  A group that does not exist (`real` false:
  // the wave's list of groups has ended) is loaded all the same, from the first bytes of every array (one cache line
  // per instruction, nothing of it is used: any bytes are valid table indices).  With loads that are only issued
  // under a condition, the number of loads behind a given one depends on the path, the compiler's wait counts
  // take the smallest, and every wait for a group's bytes becomes a wait for all loads in flight, the groups
  // requested ahead included.
  auto load_group = [&](int tg, bool real, Regs& G) {
    int64_t kbase = 0, vbase = 0, mgrp = 0;  // wave-uniform
    if (real) {
      group_bases(tg, kbase, vbase);
      mgrp = mean_base + shift_group(tg);
    }
    const uint32_t lco = real ? lane_code_off : 0u, noff = real ? norm_off : 0u, lx4 = real ? lane_x4 : 0u;
    const uint32_t ln = real ? (uint32_t)lane : 0u;
    const unsigned char* kp = kc.codes + kbase * NSV + lco;
    const unsigned char* vp = vc.codes + vbase * NSV + lco;
#pragma unroll
    for (int w4 = 0; w4 < CW / 4; ++w4) {
      const uint4 kv4 = reinterpret_cast<const uint4*>(kp)[w4];
      const uint4 vv4 = reinterpret_cast<const uint4*>(vp)[w4];
      G.kc[4 * w4] = kv4.x, G.kc[4 * w4 + 1] = kv4.y, G.kc[4 * w4 + 2] = kv4.z, G.kc[4 * w4 + 3] = kv4.w;
      G.vc[4 * w4] = vv4.x, G.vc[4 * w4 + 1] = vv4.y, G.vc[4 * w4 + 2] = vv4.z, G.vc[4 * w4 + 3] = vv4.w;
    }
    if constexpr (DQ) {
      // (kbase, vbase are multiples of 64: one norm record per 64-token block of the buffer)
      const unsigned char* kr = reinterpret_cast<const unsigned char*>(kc.norms) + (kbase >> 6) * kDqNormRec;
      const unsigned char* vr = reinterpret_cast<const unsigned char*>(vc.norms) + (vbase >> 6) * kDqNormRec;
      const uint32_t tok0 = noff >> 2;  // the lane's first token of the group (a multiple of 4)
      const uint2 ka = *reinterpret_cast<const uint2*>(kr + 2 * tok0), va = *reinterpret_cast<const uint2*>(vr + 2 * tok0);
      G.nk = make_uint4(ka.x, ka.y, *reinterpret_cast<const uint16_t*>(kr + kDqNormCodes + (tok0 >> 1)),
                        *reinterpret_cast<const uint32_t*>(kr + kDqNormPar));
      G.nv = make_uint4(va.x, va.y, *reinterpret_cast<const uint16_t*>(vr + kDqNormCodes + (tok0 >> 1)),
                        *reinterpret_cast<const uint32_t*>(vr + kDqNormPar));
      const int64_t mo = mgrp * kDqMeanRec;
      const unsigned char* km = reinterpret_cast<const unsigned char*>(kc.means) + mo;
      const unsigned char* vm = reinterpret_cast<const unsigned char*>(vc.means) + mo;
      G.ok = km[ln], G.ov = vm[ln];
      G.okp = *reinterpret_cast<const uint32_t*>(km + kDqMeanPar + 4 * (ln >> 4));
      G.ovp = *reinterpret_cast<const uint32_t*>(vm + kDqMeanPar + 4 * (ln >> 4));
    } else {
      G.nk = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(kc.norms + kbase) + noff);
      G.nv = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(vc.norms + vbase) + noff);
      const int64_t mo = mgrp * kHeadDim;
      G.ok = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const unsigned char*>(kc.means + mo) + lx4);
      G.ov = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const unsigned char*>(vc.means + mo) + lx4);
    }
  };
  // the lane's two channels of a Shift vector from its stored words
  auto mean_pair = [&](uint32_t w, uint32_t par, float& o0, float& o1) {
    if constexpr (DQ) {
      o0 = dq_level(par, w & 15u), o1 = dq_level(par, (w >> 4) & 15u);
    } else {
      o0 = half_lo_f(w), o1 = half_hi_f(w);
    }
  };

  int len, n_live, t1, n_grp, first_run = 0;
  bool res_here;  // this segment holds the unit's last group: it takes the residual rows
  if constexpr (FLAT) {
    len = len_cur;
    const int ng = max(1, (len + 63) >> 6);
    const int take_slots = min(ng + kSegCost - seg_g, run_end - run_pos);
    const int g0 = max(seg_g - kSegCost, 0), g1 = max(seg_g + take_slots - kSegCost, 0);  // the segment's groups
    if (g1 == g0) break;  // the run ends inside the unit's cost slots (all waves alike, no barrier pending)
    const int unit_pos = run_pos - seg_g + kSegCost;  // list position of the unit's first group
    first_run = unit_pos / run_q;
    n_live = (unit_pos + ng - 1) / run_q - first_run + 1;  // runs that hold groups of this unit
    split = (int)blockIdx.x - first_run;
    t0 = g0 << 6;
    t1 = min(len, g1 << 6);
    res_here = g1 == ng;
    mean_base = (int64_t)(b * hkv + h) * g.n_groups_max;
    // advance to the next segment's start (used at the end of the pass)
    run_pos += take_slots;
    seg_g = 0;  // (a run that goes on goes on with the next unit)
  }
  const int hq0 = h * (g.n_q_heads / hkv) + head_off;
  // waves 0..3 rotate one query head each (the others load a valid row that they do not use)
  auto q_row = [&](int bb, int hh0) {
    return *reinterpret_cast<const __half2*>(q + (int64_t)(bb * g.n_q_heads + hh0 + min(wave & 3, r - 1)) * kHeadDim +
                                             2 * lane);
  };
  auto mean_row_k = [&](int64_t base, int grp, uint32_t& w, uint32_t& par) {
    if constexpr (DQ) {
      const unsigned char* km = reinterpret_cast<const unsigned char*>(kc.means) + (base + grp) * kDqMeanRec;
      w = km[lane];
      par = *reinterpret_cast<const uint32_t*>(km + kDqMeanPar + 4 * (lane >> 4));
    } else {
      w = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const unsigned char*>(kc.means + (base + grp) * kHeadDim) +
                                             lane_x4);
      par = 0u;
    }
  };
  // the split's first Shift group: its q . o^k is formed once per workgroup (waves 4..7, one head each)
  const int grp_first = shift_group(min(t0, cap_tokens - 64));
  __half2 q2_raw = q2_next;
  uint32_t ok_first = okf_next, okp_first = okfp_next;
  if (!FLAT || first_segment) {
    q2_raw = q_row(b, hq0);
    mean_row_k(mean_base, grp_first, ok_first, okp_first);
  }
  if constexpr (FLAT) {
    // the unit after this one (if the run goes on, this segment ends its unit and the next begins one)
    nb = b, nh = h;
    if (run_pos < run_end && ++nh == hkv) {
      nh = 0;
      ++nb;
    }
    len_cur = seq_lens[nb];
    q2_next = q_row(nb, nh * (g.n_q_heads / hkv) + head_off);
    mean_row_k((int64_t)(nb * hkv + nh) * g.n_groups_max, 0, okf_next, okfp_next);
  }
  // (the three small loads stay ahead of the bulk ones: the waits for them then leave every later load in flight)
  __builtin_amdgcn_sched_barrier(0);
  Regs S0, S1, S2;  // each is loaded before it is read (with the bytes of a group that exists, or with any bytes)
  if constexpr (!FLAT) {
    // contiguous caches: the wave's first group is in bounds whatever the sequence length is (clamped into
    // the cache when the split lies beyond it: then it is never processed)
    if constexpr (!PAGED) load_group(min(t0 + (wave << 6), cap_tokens - 64), true, S0);  // (wslot == wave here)
    len = seq_lens[b];
    // Splits that lie wholly beyond this sequence's end have nothing to do and leave at once (a ragged batch
    // is launched with the split count of its longest sequence); the others know how many of them there
    // are.  A sequence without coded tokens keeps split 0 (it may still have residual rows).
    n_live = len > 0 ? (len - 1) / per + 1 : 1;
    if (split >= n_live) return;
    t1 = min(len, t0 + per);
    res_here = split == n_live - 1;
  }
  n_grp = (t1 > t0) ? (t1 - t0 + 63) >> 6 : 0;  // 64-token groups of this segment
  // FLAT: waves 4..7 take the segment's first groups: they are the ones that come out of the previous
  // segment early (waves 0..3 merge it), and a short segment then does not wait for the late ones
  const int wslot = FLAT ? (wave + 4) & 7 : wave;
  if constexpr (PAGED || FLAT) load_group(t0 + (wslot << 6), wslot < n_grp, S0);
  // ---- prologue: codebook table, query operands --------------------------------------------------
  if constexpr (!FLAT) fill_table();
  if (wave < 4) {  // d1: wave w rotates head w (zeros for a head that this launch does not have)
    const bool has_head = wave < r;
    const float x0 = has_head ? __low2float(q2_raw) : 0.f, x1 = has_head ? __high2float(q2_raw) : 0.f;
    const uint32_t e2 = wave * 128 + 2 * lane;  // element index of the pair in a [4][128] array
    {
      lds_write64(SM::kQorig + e2 * 4, u2v{__float_as_uint(x0), __float_as_uint(x1)});
      const float u0 = x0 * scale_log2e, u1 = x1 * scale_log2e;
      const _Float16 h0 = (_Float16)u0, h1 = (_Float16)u1;
      lds_write32(SM::kUhi + e2 * 2, __builtin_bit_cast(uint32_t, h2v{h0, h1}));
      lds_write32(SM::kUlo + e2 * 2,
                  __builtin_bit_cast(uint32_t, h2v{(_Float16)(u0 - (float)h0), (_Float16)(u1 - (float)h1)}));
    }
    float y0 = x0 + x1, y1 = x0 - x1;
    static_for<6>([&](auto kc_) {  // lane bit k <-> element bit k + 1
      constexpr int m = 1 << decltype(kc_)::value;
      const float p0 = xor_reg<m>(y0), p1 = xor_reg<m>(y1);
      const bool upper = (lane & m) != 0;
      y0 = upper ? p0 - y0 : y0 + p0;
      y1 = upper ? p1 - y1 : y1 + p1;
    });
    const float qscale = (float)kInvSqrtD * scale_log2e;
    y0 *= qscale, y1 *= qscale;
    const _Float16 h0 = (_Float16)y0, h1 = (_Float16)y1;
    lds_write32(SM::kQhi + e2 * 2, __builtin_bit_cast(uint32_t, h2v{h0, h1}));
    lds_write32(SM::kQlo + e2 * 2,
                __builtin_bit_cast(uint32_t, h2v{(_Float16)(y0 - (float)h0), (_Float16)(y1 - (float)h1)}));
  } else {
    if (first_segment && wave == 4 && lane < 32) lds_write32(SM::kZero + lane * 4, 0u);
    const int hh = wave - 4;  // this wave loaded the query of head wave & 3 = hh
    const float x0 = hh < r ? __low2float(q2_raw) : 0.f, x1 = hh < r ? __high2float(q2_raw) : 0.f;
    float of0, of1;
    mean_pair(ok_first, okp_first, of0, of1);
    const float d = wave_sum_all(x0 * of0 + x1 * of1);
    if (lane == 0) lds_write32(SM::kQoFirst + hh * 4, __float_as_uint(d * scale_log2e));
  }
  __builtin_amdgcn_sched_barrier(0);
  // residual (Sec. 3.2): wave w < 4 of the last live split takes rows [16 w, 16 w + 16); a load instruction
  // covers four consecutive rows (16 lanes x 16 bytes each); rows beyond the capacity are clamped and masked later
  const bool res_wave = res.k != nullptr && res_here && wave < 4;
  uint4 rk[4], rv[4];
  int res_len = 0;
  auto load_residual_rows = [&]() {
    const int64_t unit_row = (int64_t)(b * g.n_kv_heads + h) * res.capacity;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = min(16 * wave + 4 * u + (lane >> 4), res.capacity - 1);
      rk[u] = *reinterpret_cast<const uint4*>(res.k + (unit_row + row) * kHeadDim + (lane & 15) * 8);
      rv[u] = *reinterpret_cast<const uint4*>(res.v + (unit_row + row) * kHeadDim + (lane & 15) * 8);
    }
  };
  if (res_wave) {
    // (the persistent instance fetches the rows where it stages them: thirty-two registers held from here
    // to there do not fit beside its other state; fetching and staging them at the segment's start through
    // waves 4..7, which reach a segment first, was measured and is no faster)
    if constexpr (!FLAT) load_residual_rows();
    res_len = res.lens[b];
  }
  // The wave's second group goes out behind the first ones of all waves; every later group is requested when
  // the one before it is about to be needed (see process_group).  The compute unit's address pipeline takes
  // about 28 cycles per 1 KiB load instruction and a wave blocks at a load that cannot be accepted yet: a wave
  // that asks for more at once sits at its load instructions while the data of its first group is already in
  // its registers.  The per-split instance asks for the second group behind the first barrier and the residual
  // tile (the barrier then does not wait for eight waves' worth of load issue: 15.55 -> 15.17 us on the
  // 8 x 8192-token shape; behind the tile: 14.66 -> 14.38 us); the persistent instance, whose segments start
  // cold, in front of the barrier.
  if constexpr (FLAT) load_group(t0 + ((wslot + NW) << 6), wslot + NW < n_grp, S1);
  __syncthreads();
  if constexpr (FLAT) {
    // segments are short and start cold: three groups per wave go out before the first is used, and the set
    // that a group leaves takes the group three rounds on (see process_group)
    load_group(t0 + ((wslot + 2 * NW) << 6), wslot + 2 * NW < n_grp, S2);
  }

  // B operands of the score contraction (see the header): for tile parity p and k-step s the lane's eight
  // k-slots are channels [32 c + 8 s, +8) of head n % 4: hi part if n / 4 == p, lo part if n / 4 == p + 2,
  // zero otherwise
  const int nu = n16 >> 2;
  auto operand_addr = [&](int parity, uint32_t hi_arr, uint32_t lo_arr) -> uint32_t {
    const uint32_t off = head * 256 + rho * 64;
    return nu == parity ? hi_arr + off : nu == parity + 2 ? lo_arr + off : (uint32_t)SM::kZero;
  };
  h8 P0[4], P1[4];
  {
    const uint32_t a0 = operand_addr(0, SM::kQhi, SM::kQlo), a1 = operand_addr(1, SM::kQhi, SM::kQlo);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      P0[s] = __builtin_bit_cast(h8, lds_read128(a0 + 16 * s));
      P1[s] = __builtin_bit_cast(h8, lds_read128(a1 + 16 * s));
    }
  }

  // ---- per-lane state: one head (lane % 4), partial sums over the lane's tokens -----------------
  float m_run = -INFINITY, l_run = 0.f, beta = 0.f, cf = 1.f, qo = 0.f;
  float a_run = 0.f, w_scale = 0.f;  // A (power of two >= every a^v so far; 0 = none yet) and 2^10 / A
  f4 acc[8];                         // out_rot partial sums: component = head, see the epilogue for the channel
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = f4{0.f, 0.f, 0.f, 0.f};
  float accm[4][2];  // mean-vector term, channels 2 lane, 2 lane + 1 of the four heads
#pragma unroll
  for (int i = 0; i < 4; ++i) accm[i][0] = accm[i][1] = 0.f;
  int cur_group = -1;
  float ov0 = 0.f, ov1 = 0.f;
  const uint32_t laneoff = (SUB == 4) ? (lane & 31) * 8 : (lane & 15) * 16;  // key-side gathers
  const uint32_t laneoff_v0 = (lane & 31) * 8, laneoff_v1 = laneoff_v0 ^ 8;  // value-side 8-byte gathers

  auto half_lo = [](uint32_t u) -> float { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu)); };
  auto half_hi = [](uint32_t u) -> float { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); };

  // mean-vector term of the Shift group that just ended: accm = accm * cf + (sum of beta) * o^v
  auto flush_group = [&]() {
    const float bs = head_sum(beta);
    const float bsum[4] = {quad_bcast<0>(bs), quad_bcast<1>(bs), quad_bcast<2>(bs), quad_bcast<3>(bs)};
    const float cfh[4] = {quad_bcast<0>(cf), quad_bcast<1>(cf), quad_bcast<2>(cf), quad_bcast<3>(cf)};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      accm[i][0] = accm[i][0] * cfh[i] + bsum[i] * ov0;
      accm[i][1] = accm[i][1] * cfh[i] + bsum[i] * ov1;
    }
    beta = 0.f;
    cf = 1.f;
  };

  // d3/d4 for the lane's four tokens; returns the fp16 weights p a^v 2^10 / A as the value-side A operand.
  // Masked tokens (valid[k] false) must come in with finite sc and zero ak, bk, av, bv.
  auto softmax_step = [&](const float (&sc)[4], const bool (&valid)[4], bool all_valid, const float (&ak)[4],
                          const float (&bk)[4], const float (&av_in)[4], const float (&bv_in)[4]) -> h4 {
    float s[4];
    const float (&av)[4] = av_in;
    const float (&bv)[4] = bv_in;
#pragma unroll
    for (int k = 0; k < 4; ++k) s[k] = fmaf(ak[k], sc[k], bk[k] * qo);
    if (!all_valid) {  // wave-uniform
#pragma unroll
      for (int k = 0; k < 4; ++k) s[k] = valid[k] ? s[k] : -INFINITY;
    }
    const float smax = max3f(s[0], s[1], max2f(s[2], s[3]));
    const float amax = max3f(av[0], av[1], max2f(av[2], av[3]));
    const bool need = (smax - m_run > kLazyMaxLog2) || (amax > a_run);
    if (__any(need)) {
      const float m_new = max2f(m_run, head_max(smax));
      const float corr = (m_run == -INFINITY) ? 0.f : fast_exp2(m_run - m_new);
      l_run *= corr, beta *= corr, cf *= corr;
      m_run = m_new;
      // A: the next power of two >= the largest a^v of the wave (kept once it is large enough)
      const float amax_w = wave_max_all(amax);
      float a_new = a_run;
      if (amax_w > a_run) a_new = __uint_as_float((__float_as_uint(amax_w) + 0x007fffffu) & 0x7f800000u);
      const float a_inv = (a_new > 0.f) ? __builtin_amdgcn_rcpf(a_new) : 0.f;  // exact: a power of two
      const float a_ratio = a_run * a_inv;
      a_run = a_new;
      w_scale = kWeightScale * a_inv;
      const f4 c4 = {quad_bcast<0>(corr) * a_ratio, quad_bcast<1>(corr) * a_ratio, quad_bcast<2>(corr) * a_ratio,
                     quad_bcast<3>(corr) * a_ratio};
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] *= c4;
    }
    float w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float p = fast_exp2(s[k] - m_run);  // 0 for masked tokens
      l_run += p;
      beta = fmaf(p, bv[k], beta);
      w[k] = p * (av[k] * w_scale);
    }
    const h2v w01 = __builtin_convertvector(f2v{w[0], w[1]}, h2v), w23 = __builtin_convertvector(f2v{w[2], w[3]}, h2v);
    return h4{w01[0], w01[1], w23[0], w23[1]};
  };

  // The wave's sums over its four 16-lane groups: acc[X] of lane (rho, m, e) is a partial sum over the
  // tokens of group rho.  Two lane-swap rounds add the groups: afterwards red[j][head] of lane (rho, m, e)
  // is the wave's sum for accumulator X = j + 2 (rho & 1) + 4 (rho >> 1), times `factor`.
  auto reduce_acc = [&](float factor, float (&red)[2][4]) {
    // the swaps read registers that matrix instructions wrote: nothing may move across this point, and the
    // longest matrix instruction has drained after sixteen idle cycles
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    float red4[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float a = acc[x][i], b = acc[x + 4][i];
        lane_swap32(a, b);
        red4[x][i] = a + b;
      }
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float a = red4[x][i], b = red4[x + 2][i];
        lane_swap16(a, b);
        red[x][i] = (a + b) * factor;
      }
  };
  const int m_res = n16 >> 2, e_res = n16 & 3;  // value-side result lane: block m, column e
  const uint32_t mbase = SM::kMerge + wave * SM::kMergeWave;

  // ---- residual: one 16-token tile of fp16 rows per wave, before the wave's coded groups -----------
  // fp16 key rows are the A operand as they are, the B operand is the UNROTATED query, and the value rows
  // accumulate in the original domain: their sum becomes the start value of the mean-vector term.
  if (res_wave) {
    const int rl = min(res_len, res.capacity);
    if (rl > 16 * wave) {  // wave-uniform
      const uint32_t sk = SM::kRes + wave * SM::kResWave, sv = sk + 16 * SM::kResKStride;
      if constexpr (FLAT) load_residual_rows();
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int row = 4 * u + (lane >> 4);  // row of the tile; rows past the valid count are stored as zeros
        const bool live = 16 * wave + row < rl;
        const u4v kx = live ? u4v{rk[u].x, rk[u].y, rk[u].z, rk[u].w} : u4v{0u, 0u, 0u, 0u};
        const u4v vx = live ? u4v{rv[u].x, rv[u].y, rv[u].z, rv[u].w} : u4v{0u, 0u, 0u, 0u};
        lds_write128(sk + row * SM::kResKStride + (lane & 15) * 16, kx);
        lds_write64(sv + row * SM::kResVStride + (lane & 15) * 16, u2v{vx.x, vx.y});
        lds_write64(sv + row * SM::kResVStride + (lane & 15) * 16 + 8, u2v{vx.z, vx.w});
      }
      // written and read by different lanes of this one wave
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const int par = wave & 1;
      const uint32_t ua = operand_addr(par, SM::kUhi, SM::kUlo);
      f4 D = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        // row = token n of the tile, channels [32 rho + 8 s, +8)
        const h8 A = __builtin_bit_cast(h8, lds_read128(sk + n16 * SM::kResKStride + rho * 64 + s * 16));
        const h8 B = __builtin_bit_cast(h8, lds_read128(ua + 16 * s));
        D = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, B, D, 0, 0, 0);
      }
      // hi + lo columns; the lanes of tile `wave` (n / 4 == wave) hold its scores, all others are masked
      float sc[4];
      bool valid[4];
      const float zero[4] = {0.f, 0.f, 0.f, 0.f};
      float one[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        sc[k] = D[k] + dpp_mov<0x128>(D[k]);
        valid[k] = tile_of_lane == wave && (16 * wave + 4 * rho + k) < rl;
        one[k] = valid[k] ? 1.f : 0.f;
      }
      qo = 0.f;
      const h4 wop = softmax_step(sc, valid, false, one, zero, one, zero);
      // value rows: source lane (rho, k = n / 4, m = n % 4) reads token 4 rho + k of the tile, channels
      // [4 (4 X + m), +4); the transposing read hands lane (rho, m, e) four tokens of channel 16 X + 4 m + e
      const uint32_t vrow = sv + (4 * rho + (n16 >> 2)) * SM::kResVStride + (n16 & 3) * 8;
      static_for<4>([&](auto tc) {
        constexpr int T = decltype(tc)::value;
        if (wave == T) {  // `abid` is an immediate
          static_for<8>([&](auto xc) {
            constexpr int X = decltype(xc)::value;
            acc[X] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, lds_tr64(vrow + X * 32), acc[X], 2, T, 0);
          });
        }
      });
      // the sums change domain: through the wave's own merge slot into the mean-term registers
      float red[2][4];
      reduce_acc(a_run * (1.0f / kWeightScale), red);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int ch = 16 * (j + 2 * (rho & 1) + 4 * (rho >> 1)) + 4 * m_res + e_res;
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_write32(mbase + 2048 + (i * 128 + ch) * 4, __float_as_uint(red[j][i]));
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const u2v v2 = lds_read64(mbase + 2048 + (i * 128 + 2 * lane) * 4);
        accm[i][0] = __uint_as_float(v2.x), accm[i][1] = __uint_as_float(v2.y);
      }
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] = f4{0.f, 0.f, 0.f, 0.f};
      cf = 1.f;
    }
  }
  // (per-split instance: the wave's second group, see above; behind the residual tile, which needs no loads, so
  // that a wave with a tile asks out of the way of the other waves' load issue)
  if constexpr (!FLAT) load_group(t0 + ((wslot + NW) << 6), wslot + NW < n_grp, S1);

  // Gathers and contractions of one group, in batches.  Key side: sixteen matrix instructions in four
  // batches of four (tiles (0, 2) or (1, 3) x two k-steps, so that consecutive instructions alternate
  // between the two accumulators).  Value side: one batch per tile, eight transposed operands
  // (SUB = 4: sub-vectors 4 X + m; SUB = 8: sub-vectors 4 x + m as two halves, accumulator 2 x + hf).
  auto k_gather = [&](auto bc, const Regs& G, h8 (&A)[4]) {  // A[2 * sp + tp]: tile 2 tp + (B & 1), k-step 2 (B >> 1) + sp
    constexpr int B = decltype(bc)::value;
    static_for<4>([&](auto ec) {
      constexpr int E = decltype(ec)::value;
      constexpr int T = 2 * (E & 1) + (B & 1), S = 2 * (B >> 1) + (E >> 1);
      if constexpr (SUB == 4) {
        const uint32_t w = G.kc[2 * T + (S >> 1)];
        const u2v c0 = lds_read64(table_addr<2 * (S & 1)>(w, laneoff));
        const u2v c1 = lds_read64(table_addr<2 * (S & 1) + 1>(w, laneoff));
        A[E] = __builtin_bit_cast(h8, u4v{c0.x, c0.y, c1.x, c1.y});
      } else {
        A[E] = __builtin_bit_cast(h8, lds_read128(table_addr<S>(G.kc[T], laneoff)));
      }
    });
  };
  auto k_contract = [&](auto bc, const h8 (&A)[4], f4& D0, f4& D1) {
    constexpr int B = decltype(bc)::value;
    static_for<4>([&](auto ec) {
      constexpr int E = decltype(ec)::value;
      constexpr int S = 2 * (B >> 1) + (E >> 1);
      if constexpr ((E & 1) == 0)  // tiles 0, 1 -> D0; tiles 2, 3 -> D1
        D0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[E], (B & 1) ? P1[S] : P0[S], D0, 0, 0, 0);
      else
        D1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[E], (B & 1) ? P1[S] : P0[S], D1, 0, 0, 0);
    });
  };
  auto v_gather = [&](auto tc, const Regs& G, h4 (&Bv)[8]) {
    constexpr int T = decltype(tc)::value;
    static_for<8>([&](auto xc) {
      constexpr int X = decltype(xc)::value;
      if constexpr (SUB == 4)
        Bv[X] = lds_tr64(table_addr<X & 3>(G.vc[2 * T + (X >> 2)], laneoff_v0));
      else
        Bv[X] = lds_tr64(table_addr<(X >> 1)>(G.vc[T], (X & 1) ? laneoff_v1 : laneoff_v0));
    });
  };
  auto v_contract = [&](auto tc, const h4 (&Bv)[8], const h4& wop) {
    constexpr int T = decltype(tc)::value;
    static_for<8>([&](auto xc) {
      constexpr int X = decltype(xc)::value;
      acc[X] = __builtin_amdgcn_mfma_f32_4x4x4f16(wop, Bv[X], acc[X], 2, T, 0);
    });
  };
  constexpr std::integral_constant<int, 0> c0{};
  constexpr std::integral_constant<int, 1> c1{};
  constexpr std::integral_constant<int, 2> c2{};
  constexpr std::integral_constant<int, 3> c3{};

  // One group: scores, softmax, value accumulation.  `G` holds the group's bytes, KA / KB the first two
  // key-side gather batches of it (issued while the previous group's value side was running); they are
  // refilled for `Gn`, the wave's next group, before this group's last matrix instructions are issued.
  // A gather batch is always issued two batches ahead of its matrix instructions; scheduling barriers keep
  // the compiler from sinking the gathers next to their uses, which would expose the LDS latency at
  // every one of the 48 matrix instructions of a group.
  // (inside a stage the matrix instructions go first: the operands they consume are dead before the next
  // gathers land, so a later batch can take over an earlier one's registers)
  h8 KA[4], KB[4];
  auto process_group = [&](int gi, Regs& G, const Regs& Gn, Regs& Gnn) {
    const int tg = t0 + (gi << 6);
    // Shift group bookkeeping (wave-uniform)
    const int grp = shift_group(tg);
    if (grp != cur_group) {
      if (cur_group >= 0) flush_group();
      if (grp == grp_first) {
        qo = lds_read32f(SM::kQoFirst + head * 4);
      } else {
        float o0, o1;
        mean_pair(G.ok, G.okp, o0, o1);
        float qd[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const u2v q2u = lds_read64(SM::kQorig + (i * 128 + 2 * lane) * 4);
          qd[i] = wave_sum_all(__uint_as_float(q2u.x) * o0 + __uint_as_float(q2u.y) * o1);
        }
        const float lo01 = (head & 1) ? qd[1] : qd[0], hi23 = (head & 1) ? qd[3] : qd[2];
        qo = ((head & 2) ? hi23 : lo01) * scale_log2e;
      }
      mean_pair(G.ov, G.ovp, ov0, ov1);
      cur_group = grp;
    }
    // d2/d3: HT(q) . C[codes] of the group's 64 tokens, four heads
    f4 D0 = {0.f, 0.f, 0.f, 0.f}, D1 = {0.f, 0.f, 0.f, 0.f};
    h8 KC[4], KD[4];
    h4 VA[8], VB[8], VC[8], VD[8];
    __builtin_amdgcn_sched_barrier(0);
    k_contract(c0, KA, D0, D1);
    __builtin_amdgcn_sched_barrier(0);
    k_gather(c2, G, KC);
    __builtin_amdgcn_sched_barrier(0);
    k_contract(c1, KB, D0, D1);
    __builtin_amdgcn_sched_barrier(0);
    k_gather(c3, G, KD);
    __builtin_amdgcn_sched_barrier(0);
    k_contract(c2, KC, D0, D1);
    __builtin_amdgcn_sched_barrier(0);
    v_gather(c0, G, VA);  // the first value-side gathers fly during the softmax arithmetic
    __builtin_amdgcn_sched_barrier(0);
    k_contract(c3, KD, D0, D1);
    __builtin_amdgcn_sched_barrier(0);
    v_gather(c1, G, VB);
    __builtin_amdgcn_sched_barrier(0);
    // hi + lo columns: lanes n < 8 take tiles 0, 1 from D0, lanes n >= 8 tiles 2, 3 from D1
    float sc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float x = D0[k] + dpp_mov<0x128>(D0[k]);
      const float y = D1[k] + dpp_mov<0x128>(D1[k]);
      sc[k] = (n16 < 8) ? x : y;
    }
    const bool all_valid = (tg + 64 <= t1);
    bool valid[4] = {true, true, true, true};
    if (!all_valid) {  // wave-uniform: only a sequence's last group has masked tokens (their bytes may be anything)
      const int tb0 = tg + 16 * tile_of_lane + 4 * rho;  // the lane's first token
#pragma unroll
      for (int k = 0; k < 4; ++k) valid[k] = (tb0 + k) < t1;
    }
    float ak[4], bk[4], av[4], bv[4];
    if constexpr (DQ) {  // b = min + step * code, a = b * a'
      const float apk[4] = {half_lo(G.nk.x), half_hi(G.nk.x), half_lo(G.nk.y), half_hi(G.nk.y)};
      const float apv[4] = {half_lo(G.nv.x), half_hi(G.nv.x), half_lo(G.nv.y), half_hi(G.nv.y)};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float b_k = dq_level(G.nk.w, (G.nk.z >> (4 * k)) & 15u), b_v = dq_level(G.nv.w, (G.nv.z >> (4 * k)) & 15u);
        bk[k] = valid[k] ? b_k : 0.f, ak[k] = valid[k] ? b_k * apk[k] : 0.f;
        bv[k] = valid[k] ? b_v : 0.f, av[k] = valid[k] ? b_v * apv[k] : 0.f;
      }
    } else {
      uint32_t nkw[4] = {G.nk.x, G.nk.y, G.nk.z, G.nk.w}, nvw[4] = {G.nv.x, G.nv.y, G.nv.z, G.nv.w};
      if (!all_valid) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          nkw[k] = valid[k] ? nkw[k] : 0u;
          nvw[k] = valid[k] ? nvw[k] : 0u;
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        ak[k] = half_lo(nkw[k]), bk[k] = half_hi(nkw[k]);
        av[k] = half_lo(nvw[k]), bv[k] = half_hi(nvw[k]);
      }
    }
    const h4 wop = softmax_step(sc, valid, all_valid, ak, bk, av, bv);

    // d5: out_rot[head][channel] += sum over tokens of weight * codeword channel
    __builtin_amdgcn_sched_barrier(0);
    v_contract(c0, VA, wop);
    __builtin_amdgcn_sched_barrier(0);
    v_gather(c2, G, VC);
    __builtin_amdgcn_sched_barrier(0);
    v_contract(c1, VB, wop);
    __builtin_amdgcn_sched_barrier(0);
    v_gather(c3, G, VD);
    __builtin_amdgcn_sched_barrier(0);
    // the group after the next one: requested just before the next one's bytes are first needed (below)
    if constexpr (FLAT)  // (this group's bytes have all been used by now)
      load_group(t0 + ((gi + 3 * NW) << 6), gi + 3 * NW < n_grp, G);
    else
      load_group(t0 + ((gi + 2 * NW) << 6), gi + 2 * NW < n_grp, Gnn);
    __builtin_amdgcn_sched_barrier(0);
    v_contract(c2, VC, wop);
    __builtin_amdgcn_sched_barrier(0);
    k_gather(c0, Gn, KA);  // (any bytes are valid table indices: harmless when there is no next group)
    __builtin_amdgcn_sched_barrier(0);
    v_contract(c3, VD, wop);
    __builtin_amdgcn_sched_barrier(0);
    k_gather(c1, Gn, KB);
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- main loop: this wave's groups wave, wave + NW, ...; three register sets rotate (in use, next, in flight) ----
  if (wslot < n_grp) {
    int gi = wslot;
    k_gather(c0, S0, KA);
    k_gather(c1, S0, KB);
    while (true) {
      process_group(gi, S0, S1, S2);
      gi += NW;
      if (gi >= n_grp) break;
      process_group(gi, S1, S2, S0);
      gi += NW;
      if (gi >= n_grp) break;
      process_group(gi, S2, S0, S1);
      gi += NW;
      if (gi >= n_grp) break;
    }
  }
  if (cur_group >= 0) flush_group();
  // the window of the unit that the next segment begins (pages 0..63), back before that segment asks for it
  if constexpr (FLAT && PAGED) load_window(nb, 0, nwin_k, nwin_v);

  // ---- epilogue: this wave's sums -> its merge slot ------------------------------------------------
  {
    float red[2][4];
    reduce_acc(a_run * (1.0f / kWeightScale), red);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int X = j + 2 * (rho & 1) + 4 * (rho >> 1);
      int ch;
      if constexpr (SUB == 4)
        ch = 16 * X + 4 * m_res + e_res;
      else  // X = 2 x + hf: sub-vector 4 x + m, half hf ^ (m & 1) (odd lanes gather the other half first)
        ch = 8 * (4 * (X >> 1) + m_res) + 4 * ((X & 1) ^ (m_res & 1)) + e_res;
#pragma unroll
      for (int i = 0; i < 4; ++i) lds_write32(mbase + (i * 128 + ch) * 4, __float_as_uint(red[j][i]));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      lds_write64(mbase + 2048 + (i * 128 + 2 * lane) * 4, u2v{__float_as_uint(accm[i][0]), __float_as_uint(accm[i][1])});
    const float l_tot = head_sum(l_run);
    if (lane < 4) lds_write64(mbase + 4096 + lane * 8, u2v{__float_as_uint(m_run), __float_as_uint(l_tot)});
  }
  __syncthreads();

  // ---- merge the waves: wave i takes head i, a lane channels 2 lane, 2 lane + 1 ------------------
  [&]() {
  if (wave >= r) return;
  const int hh = wave;
  float M = -INFINITY, L = 0.f, x0 = 0.f, x1 = 0.f, mm0 = 0.f, mm1 = 0.f;
  {
    float mw[NW], lw[NW];
    f2v rw[NW], qw[NW];
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      const uint32_t mb = SM::kMerge + wv * SM::kMergeWave;
      const u2v ml = lds_read64(mb + 4096 + hh * 8);
      mw[wv] = __uint_as_float(ml.x), lw[wv] = __uint_as_float(ml.y);
      rw[wv] = __builtin_bit_cast(f2v, lds_read64(mb + (hh * 128 + 2 * lane) * 4));
      qw[wv] = __builtin_bit_cast(f2v, lds_read64(mb + 2048 + (hh * 128 + 2 * lane) * 4));
    }
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) M = fmaxf(M, mw[wv]);
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      const float e = (mw[wv] == -INFINITY) ? 0.f : fast_exp2(mw[wv] - M);
      L = fmaf(e, lw[wv], L);
      x0 = fmaf(e, rw[wv][0], x0), x1 = fmaf(e, rw[wv][1], x1);
      mm0 = fmaf(e, qw[wv][0], mm0), mm1 = fmaf(e, qw[wv][1], mm1);
    }
  }

  // ---- d6: merge the splits; the last wave to arrive for this query head finishes it -------------
  if (n_live > 1) {
    // !FLAT: partial [sequence][query head][split].  FLAT: [run][slot][query head of the kv head]: slot 0 for
    // the segment that continues a unit begun in an earlier run, slot 1 for the one that begins a unit and
    // leaves its end to the next run (a run has at most one of each); run c of the unit's runs
    // first_run .. first_run + n_live - 1 therefore wrote slot 1 if c == first_run, else slot 0.
    auto partial_of = [&](int s) -> float* {
      if constexpr (FLAT)
        return partial + ((int64_t)((first_run + s) * 2 + (s == 0 ? 1 : 0)) * (g.n_q_heads / hkv) + head_off + hh) * kPartialStride;
      else
        return partial + ((int64_t)(b * g.n_q_heads + hq0 + hh) * n_splits + s) * kPartialStride;
    };
    float* P = partial_of(split);
    auto st2 = [](float* p, float lo, float hi) {  // 8-byte device-scope store (p is 8-byte aligned)
      __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                         ((unsigned long long)__float_as_uint(hi) << 32) | __float_as_uint(lo), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    };
    auto ld2 = [](const float* p) -> float2 {
      const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
      return make_float2(__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32)));
    };
    st2(P + 2 * lane, x0, x1);
    st2(P + kHeadDim + 2 * lane, mm0, mm1);
    if (lane == 0) st2(P + 2 * kHeadDim, M, L);
    // The partials are written with device-scope stores (they go through to memory: no cache holds them
    // back), the wave waits until every one has been acknowledged, and only then counts itself in; the
    // wave that reads n_live - 1 reads the other splits' partials with device-scope loads (they do not hit
    // in a cache that could hold older bytes).  The agent-scope release / acquire fences that would say
    // the same in the memory model make the compiler write back and invalidate the whole L2 around
    // the counter update: measured 7 us + 4 us per launch on the 8 x 8192-token shape.
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    int* cnt = counters + (b * g.n_q_heads + hq0 + hh) * kCounterStrideInts;
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != n_live - 1) return;
    if (lane == 0) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
    // chunks of SF splits, every load of a chunk issued before its first use (a chunk costs one trip to
    // memory); running max across chunks.  Up to eight live splits take one chunk of eight, more take chunks
    // of thirty-two (the loop's registers are free by now).
    M = -INFINITY, L = 0.f, x0 = x1 = mm0 = mm1 = 0.f;
    auto merge_chunks = [&](auto sfc) {
      constexpr int SF = decltype(sfc)::value;
      for (int s0 = 0; s0 < n_live; s0 += SF) {
        float2 pml[SF], pr[SF], pq[SF];
#pragma unroll
        for (int s = 0; s < SF; ++s) {
          pml[s] = make_float2(-INFINITY, 0.f);
          pr[s] = pq[s] = make_float2(0.f, 0.f);
          if (s0 + s < n_live) {  // uniform
            const float* ps = partial_of(s0 + s);
            pml[s] = ld2(ps + 2 * kHeadDim);
            pr[s] = ld2(ps + 2 * lane);
            pq[s] = ld2(ps + kHeadDim + 2 * lane);
          }
        }
        float Mn = M;
#pragma unroll
        for (int s = 0; s < SF; ++s) Mn = fmaxf(Mn, pml[s].x);
        if (Mn > -INFINITY) {
          const float corr = (M == -INFINITY) ? 0.f : fast_exp2(M - Mn);
          L *= corr, x0 *= corr, x1 *= corr, mm0 *= corr, mm1 *= corr;
#pragma unroll
          for (int s = 0; s < SF; ++s) {
            const float e = (s0 + s < n_live) ? fast_exp2(pml[s].x - Mn) : 0.f;
            L = fmaf(e, pml[s].y, L);
            x0 = fmaf(e, pr[s].x, x0), x1 = fmaf(e, pr[s].y, x1);
            mm0 = fmaf(e, pq[s].x, mm0), mm1 = fmaf(e, pq[s].y, mm1);
          }
          M = Mn;
        }
      }
    };
    if (n_live <= 8)
      merge_chunks(std::integral_constant<int, 8>{});
    else
      merge_chunks(std::integral_constant<int, 32>{});
  }
  // one inverse Hadamard per head (H is its own inverse), across the wave's lanes in registers
  {
    const float a0 = x0 + x1, a1 = x0 - x1;
    x0 = a0, x1 = a1;
  }
  static_for<6>([&](auto kc_) {
    constexpr int m = 1 << decltype(kc_)::value;
    const float p0 = xor_reg<m>(x0), p1 = xor_reg<m>(x1);
    const bool upper = (lane & m) != 0;
    x0 = upper ? p0 - x0 : x0 + p0;
    x1 = upper ? p1 - x1 : x1 + p1;
  });
  float2 o2 = make_float2(0.f, 0.f);
  if (L > 0.f) o2 = make_float2((x0 * (float)kInvSqrtD + mm0) / L, (x1 * (float)kInvSqrtD + mm1) / L);
  *reinterpret_cast<float2*>(out + (int64_t)(b * g.n_q_heads + hq0 + hh) * kHeadDim + 2 * lane) = o2;
  }();
  if constexpr (!FLAT) break;
  if (run_pos >= run_end) break;
  b = nb, h = nh;  // the next unit (its first row and length are on their way or here)
  first_segment = false;
  if constexpr (PAGED) win0 = 0, win_k = nwin_k, win_v = nwin_v;
  }  // segments
}


template <int SUB, int NW, bool POW2, bool PAGED, bool FLAT, bool DQ>
static int launch_one(const Geometry& g, const void* codebook, const void* q, const CacheView& kv, const CacheView& vv,
                      const int32_t* seq_lens, int batch, int max_seq_len, float scale, int n_splits, void* workspace,
                      size_t counter_bytes, const ResidualView& res, int head_off, int r_pass, float* out,
                      hipStream_t stream) {
  using SM = Smem<NW>;
  const size_t smem = res.k != nullptr ? (size_t)SM::kBytesRes : (size_t)SM::kBytes;
  static const int attr_rc = [] {
    // the gathers address the codebook table by absolute LDS address: it must start at 0, i.e. the
    // kernel may not own any static LDS in front of its dynamic block
    hipFuncAttributes fa;
    const void* fn = reinterpret_cast<const void*>(dec_tile_kernel<SUB, NW, POW2, PAGED, FLAT, DQ>);
    if (hipFuncGetAttributes(&fa, fn) != hipSuccess || fa.sharedSizeBytes != 0) return (int)NSN_ERR_HIP;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SM::kBytesRes) != hipSuccess)
      return (int)NSN_ERR_HIP;
    return (int)NSN_OK;
  }();  // initialised once, thread-safe
  if (attr_rc != NSN_OK) return attr_rc;
  int* counters = static_cast<int*>(workspace);
  float* partial = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + counter_bytes);
  int per = 0;
  dim3 grid;
  if constexpr (FLAT) {
    // one workgroup per compute unit, never more runs than the workspace has partial slots for
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
      return NSN_ERR_HIP;
    const int64_t groups_max = (int64_t)batch * g.n_kv_heads * max(1, (max_seq_len + 63) / 64);
    n_splits = (int)std::min<int64_t>(std::min(n_cu, kFlatRunsMax), groups_max);
    grid = dim3(n_splits, 1, 1);
  } else {
    per = (((max_seq_len + n_splits - 1) / n_splits) + 63) & ~63;
    grid = dim3(n_splits, g.n_kv_heads, batch);
  }
  dec_tile_kernel<SUB, NW, POW2, PAGED, FLAT, DQ><<<grid, NW * 64, smem, stream>>>(
      g, (const __half*)codebook, (const __half*)q, kv, vv, seq_lens, batch, scale * 1.44269504088896340736f, n_splits,
      per, partial, counters, res, head_off, r_pass, out);
  return hipGetLastError() == hipSuccess ? NSN_OK : NSN_ERR_HIP;
}

}  // namespace tile

int decode_tile_launch(const nsn_shape& s, const void* codebook, const void* q, const nsn_cache& kc,
                       const nsn_cache& vc, const int32_t* seq_lens, int batch, int max_seq_len, float scale,
                       int n_splits, void* workspace, size_t counter_bytes, const nsn_residual* residual, float* out,
                       hipStream_t stream) {
  const Geometry g = make_geometry(s);
  ResidualView res = {nullptr, nullptr, nullptr, 0};
  if (residual)
    res = {static_cast<const __half*>(residual->k_fp16), static_cast<const __half*>(residual->v_fp16),
           residual->lens, residual->capacity};
  const CacheView kv = make_view(kc), vv = make_view(vc);
  const int r_total = s.n_q_heads / s.n_kv_heads;
  // up to four query heads per kv head in one launch; five to eight as two launches on the same stream
  for (int head_off = 0; head_off < r_total; head_off += 4) {
    const int r = min(4, r_total - head_off);
#define NSN_TILE_ARGS \
  g, codebook, q, kv, vv, seq_lens, batch, max_seq_len, scale, n_splits, workspace, counter_bytes, res, head_off, r, out, stream
    const bool pow2 = (g.group_size <= 0 || g.group_shift >= 0) && (!g.paged || g.page_shift >= 0);
    auto with_flags = [&](auto sub, auto flat, auto dq) {
      constexpr int kSub = decltype(sub)::value;
      constexpr bool kFlat = decltype(flat)::value, kDq = decltype(dq)::value;
      if (g.paged)
        return pow2 ? tile::launch_one<kSub, 8, true, true, kFlat, kDq>(NSN_TILE_ARGS)
                    : tile::launch_one<kSub, 8, false, true, kFlat, kDq>(NSN_TILE_ARGS);
      return pow2 ? tile::launch_one<kSub, 8, true, false, kFlat, kDq>(NSN_TILE_ARGS)
                  : tile::launch_one<kSub, 8, false, false, kFlat, kDq>(NSN_TILE_ARGS);
    };
    auto with_sub = [&](auto flat) {
      if (g.dq)
        return s.sub_dim == 4 ? with_flags(std::integral_constant<int, 4>{}, flat, std::true_type{})
                              : with_flags(std::integral_constant<int, 8>{}, flat, std::true_type{});
      return s.sub_dim == 4 ? with_flags(std::integral_constant<int, 4>{}, flat, std::false_type{})
                            : with_flags(std::integral_constant<int, 8>{}, flat, std::false_type{});
    };
    // n_splits == kSplitsFlat: the persistent instance that cuts the list of all groups into equal runs
    const int rc = n_splits == kSplitsFlat ? with_sub(std::true_type{}) : with_sub(std::false_type{});
#undef NSN_TILE_ARGS
    if (rc != NSN_OK) return rc;
  }
  return NSN_OK;
}

}  // namespace nsn
