// Internal declarations shared by the translation units of libsapo (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <tuple>
#include <stddef.h>

#include "../../include/sapo.h"

namespace sapo {

typedef __bf16 bf16;
typedef _Float16 f16;   // MFMA operand type: packed weights, activations, KV cache of the MFMA path

constexpr int kPageTokens = 16;
constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------
// Row -> (sequence, position) maps.  A "row" is one token being pushed through the layers.
//   block mode : rows are laid out [n_seq, T]; row m is position m % T of cache sequence
//                (m / T) * seq_stride (prefill of prompt p writes through the page table of
//                the first sibling, seq_stride = G; scoring uses seq_stride = 1).
//   decode mode: row m is sequence m at position Lp + *step - 1 (the token sampled at the
//                previous step); *step lives in device memory so that one captured graph
//                can be replayed for every step.
// Prompts of different lengths (optional): lens[p] is the length of prompt p = sequence / G.  Block rows
// at or past their prompt's length are padding: they run through the layers but leave no K/V behind;
// decode rows sit at lens[p] + *step - 1.
// ---------------------------------------------------------------------------------------
struct RowMap {
  int decode;       // 0 block, 1 decode
  int T;            // block mode: positions per sequence
  int seq_stride;   // block mode: cache-sequence stride
  int Lp;           // decode mode: prompt length
  const int* step;  // decode mode: device pointer to the current step index (>= 1)
  const int* lens;  // optional, device: prompt lengths
  int G;            // sequences per prompt (with lens)
  // decode mode, optional, device: the sequence behind each row once ended sequences have been taken out of
  // the batch (row m of the step's activations belongs to sequence slot_seq[m]); NULL: row m is sequence m
  const int* slot_seq = nullptr;
  __device__ __forceinline__ void get(int m, int& seq, int& pos) const {
    if (decode) {
      seq = slot_seq ? slot_seq[m] : m;
      pos = (lens ? lens[seq / G] : Lp) + *step - 1;
    } else {
      seq = (m / T) * seq_stride;
      pos = m % T;
    }
  }
  // does row m leave K/V in the cache?
  __device__ __forceinline__ bool keeps_kv(int m) const { return decode || !lens || (m % T) < lens[m / T]; }
};

// Paged KV cache of one layer.  K page: [Hkv][16 tokens][hd]; V page: [Hkv][hd][16 tokens]
// (V is kept token-minor so that a fixed feature's 16 tokens are contiguous).
// Element type: fp32 for fp32 models; for bf16 models the shape-generic kernels keep bf16 and the
// MFMA kernels keep IEEE half (same 2 bytes, 3 more mantissa bits: attention involves no weights,
// so its operands need not share the weights' type; values are clamped to the half range).
struct KVCache {
  void* k;                // [n_pages][Hkv][16][hd]
  void* v;                // [n_pages][Hkv][hd][16]
  const int* page_table;  // [n_cache_seq][pages_per_seq]
  int pages_per_seq;
  int n_kv_heads;
  int head_dim;
};

// ---------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------
// A pair (a, b) rotated by (cos, sin), the rounding written out - one product rounded, then one fused multiply-add -
// so that every decode kernel that rotates gives the same bits whatever the code around the expression looks like
// (left to the compiler, which product is fused depends on the instruction order it happens to pick).
__device__ __forceinline__ float rot_first(float a, float b, float c, float s) { return __builtin_fmaf(a, c, -(b * s)); }
__device__ __forceinline__ float rot_second(float a, float b, float c, float s) { return __builtin_fmaf(b, c, a * s); }
template <typename T> __device__ __forceinline__ float to_f32(T x) { return static_cast<float>(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x) { return static_cast<T>(x); }
template <> __device__ __forceinline__ f16 from_f32<f16>(float x) { return (f16)fminf(fmaxf(x, -65504.f), 65504.f); }

// The wave's index inside its workgroup as a scalar (the same for every lane, and known to the compiler as such).
// Kernels guard matrix-core instructions with conditions on it ("has this wave another k step"); with the index in
// a vector register such a guard is a lane mask, the compiler may drop the branch around a short masked block, and a
// matrix-core instruction - which ignores the lane mask - then runs on registers that hold nothing.  A scalar index
// makes the guard a real branch.
__device__ __forceinline__ int wave_index(int thread_index) { return __builtin_amdgcn_readfirstlane(thread_index >> 6); }

// The values of lanes l and l ^ 16 (l ^ 32) combined in every lane, through gfx950's lane-swap instructions
// (v_permlane16_swap / v_permlane32_swap: one vector-ALU instruction, no trip through LDS as the generic shuffle
// takes).  Both lanes of a pair combine (lower lane's value, upper lane's value) in that order.
typedef unsigned int lane_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_xor16(float x) {
  const lane_u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float max_xor32(float x) {
  const lane_u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor16(float x) {
  const lane_u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum_xor32(float x) {
  const lane_u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float wave_reduce_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_reduce_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds on a 4-word counter with a 2-word key.
struct Philox4 { uint32_t x, y, z, w; };
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return Philox4{c0, c1, c2, c3};
}

// Standard Gumbel noise from one 32-bit random word: u = (2 (x >> 9) + 1) 2^-24 is strictly
// inside (0, 1) and exact in fp32; g = -ln(-ln u).
__device__ __forceinline__ float gumbel_from_bits(uint32_t x) {
  const float u = (float)(2u * (x >> 9) + 1u) * 5.9604644775390625e-08f;
  return -logf(-logf(u));
}

// Noise for vocab entries 4*blk .. 4*blk+3 of (seed, seq, step): counter (blk, step, seq, 0),
// key = (seed low, seed high); entry v uses output word v % 4.
__device__ __forceinline__ void gumbel4(uint32_t seed_lo, uint32_t seed_hi, uint32_t seq, uint32_t step,
                                        uint32_t blk, float g[4]) {
  const Philox4 r = philox4x32_10(blk, step, seq, 0u, seed_lo, seed_hi);
  g[0] = gumbel_from_bits(r.x); g[1] = gumbel_from_bits(r.y);
  g[2] = gumbel_from_bits(r.z); g[3] = gumbel_from_bits(r.w);
}

// Running (max, sum of exp) pair of an online log-sum-exp.
struct LseAcc {
  float m, l;
  __device__ __forceinline__ void init() { m = -INFINITY; l = 0.f; }
  __device__ __forceinline__ void add(float z) {
    if (z > m) { l = l * __expf(m - z) + 1.f; m = z; } else { l += __expf(z - m); }
  }
  __device__ __forceinline__ void merge(float m2, float l2) {
    const float mn = fmaxf(m, m2);
    if (mn == -INFINITY) return;
    l = l * __expf(m - mn) + l2 * __expf(m2 - mn);
    m = mn;
  }
};

// Best perturbed score so far: larger y wins, equal y goes to the lower id.
struct BestAcc {
  float y, z; int id;
  __device__ __forceinline__ void init() { y = -INFINITY; z = 0.f; id = 0x7fffffff; }
  __device__ __forceinline__ void add(float y2, float z2, int id2) {
    if (y2 > y || (y2 == y && id2 < id)) { y = y2; z = z2; id = id2; }
  }
};

// ---------------------------------------------------------------------------------------
// Host-side launchers.  Every launcher enqueues on `st` and returns the launch's hipError_t.
// dtype: SAPO_DTYPE_F32 / SAPO_DTYPE_BF16 selects the element type T of weights/activations.
// ---------------------------------------------------------------------------------------
struct SampleParams {
  float temperature;
  uint32_t seed_lo, seed_hi;
  int max_new;            // row stride of out_tokens / out_logprobs
  const int* step;        // device: index of the token being sampled (0-based)
  const uint32_t* dyn;    // device, optional: {seed_lo, seed_hi, temperature bits} overriding the fields above
                          // (lets one captured graph serve calls that differ only in seed / temperature)
  int32_t* out_tokens;    // [S, max_new]
  float* out_logprobs;    // [S, max_new]
  // Stop token (optional): stop[0] = the token id that ends a sequence (< 0: none), stop[1] = number of
  // finished sequences, stop[2 + s] = length of sequence s once it has ended (0 while it runs).
  int* stop = nullptr;
  // Optional: arrival counter of the sampler's merge kernel.  When set, the last workgroup of the merge to
  // have read *step advances it (the step counter then needs no kernel of its own).
  int* arrivals = nullptr;
  // Optional, device: the sequence behind each row of the step (see RowMap::slot_seq).  The noise is keyed on
  // the sequence, and tokens, log-probs and lengths are written at the sequence's own rows.
  const int* slot_seq = nullptr;
  // Optional, device: a word that is non-zero once a decode step could not complete (see PersistCtl::fault).  From
  // then on the sampler emits token -1 with log-prob 0, so the failure is visible in the call's output.
  const unsigned* fault = nullptr;
  // Vocabulary size (0: unknown).  A sampled id outside [0, vocab) - what a row of NaN logits leaves behind, since no
  // score ever beats the initial one - is emitted as -1 and never used as an index.
  int vocab = 0;
};

// Optional per-kernel timing: when switched on, every launch carries two HIP events that take
// the kernel's start and end timestamps; the totals are read back per kernel symbol.  Off by
// default (the only cost is one branch per launch).
enum KernelId {
  KID_EMBED = 0, KID_RMSNORM, KID_GEMM_GENERIC, KID_ROPE_APPEND, KID_ATTN_GENERIC, KID_SWIGLU, KID_SAMPLE_ROWS,
  KID_SCORE_ROWS, KID_MISC, KID_GEMM_BIG, KID_LMHEAD_SCORE, KID_LMHEAD_SCORE_MERGE, KID_GEMM_SKINNY,
  KID_LMHEAD_SAMPLE, KID_LMHEAD_SAMPLE_MERGE, KID_DECODE_ATTN, KID_FLASH_ATTN, KID_GEMM_BIG_DECODE, KID_DECODE_LAYERS,
  KID_DECODE_ATTN_SHARED, KID_COUNT
};
extern bool g_prof_on;
// A pair of events for one profiled launch of kernel `kid` (recorded for sapo_profile_stop).
void prof_events(int kid, hipEvent_t* e0, hipEvent_t* e1);

// Every kernel launch of the library goes through here.  Normally a plain launch; while
// profiling, the launch carries two events that receive the kernel's own start and end
// timestamps (the figures a kernel trace reports, without the launch gaps around them).
template <typename... KArgs, typename... Args>
inline hipError_t launch(int kid, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t smem, hipStream_t st,
                         Args... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count mismatch");
  std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
  void* ptrs[sizeof...(KArgs) + 1];
  std::apply([&](auto&... v) { int i = 0; ((ptrs[i++] = (void*)&v), ...); }, vals);
  if (g_prof_on) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    prof_events(kid, &e0, &e1);
    return hipExtLaunchKernel((const void*)kernel, grid, block, ptrs, smem, st, e0, e1, 0);
  }
  return hipLaunchKernel((const void*)kernel, grid, block, ptrs, smem, st);
}

// The one place a sampled token is written.  A sequence that has emitted the stop token keeps
// emitting it with log-prob 0 (padding); the token returned is the one the next step embeds.
__device__ __forceinline__ int emit_token(const SampleParams& sp, int seq, int step, int token, float logprob) {
  if ((sp.fault && *sp.fault != 0u) || (sp.vocab > 0 && (unsigned)token >= (unsigned)sp.vocab)) {
    const size_t o = (size_t)seq * sp.max_new + step;
    sp.out_tokens[o] = -1;
    sp.out_logprobs[o] = 0.f;
    return 0;   // a valid id for the next step's embedding gather
  }
  if (sp.stop && sp.stop[0] >= 0) {
    int* len = sp.stop + 2 + seq;
    if (*len > 0) {
      token = sp.stop[0];
      logprob = 0.f;
    } else if (token == sp.stop[0]) {
      *len = step + 1;
      atomicAdd(sp.stop + 1, 1);
    }
  }
  const size_t o = (size_t)seq * sp.max_new + step;
  sp.out_tokens[o] = token;
  sp.out_logprobs[o] = logprob;
  return token;
}

__device__ __forceinline__ void resolve_sample_params(SampleParams& sp) {
  if (sp.dyn) {
    sp.seed_lo = sp.dyn[0];
    sp.seed_hi = sp.dyn[1];
    sp.temperature = __uint_as_float(sp.dyn[2]);
  }
}

// generic (shape-agnostic) kernels --------------------------------------------------------
hipError_t g_embed(int dtype, const int32_t* tokens, int tok_stride, const int* step, const void* embed,
                   float* h, int M, int d, hipStream_t st);
hipError_t g_rmsnorm(int dtype, const float* h, const float* gain, float eps, void* out, int M, int d,
                     const int* row_index, hipStream_t st);
enum GemmEpi { EPI_STORE_F32 = 0, EPI_ADD_F32 = 1 };
hipError_t g_gemm(int dtype, const void* A, const void* W, float* C, int M, int N, int K, int ldc, GemmEpi epi,
                  hipStream_t st);
hipError_t g_rope_append(int dtype, const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* q_out,
                         int M, int n_q_heads, hipStream_t st);
// same, with q_out and the cache in IEEE half (MFMA path)
hipError_t g_rope_append_f16(const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* q_out, int M,
                             int n_q_heads, hipStream_t st);
hipError_t g_attention(int dtype, const void* q, RowMap rm, KVCache kv, void* out, int M, int n_q_heads,
                       int max_ctx, hipStream_t st);
hipError_t g_swiglu(int dtype, const float* gu, void* act, int M, int F, hipStream_t st);
hipError_t g_sample_rows(const float* logits, int n_prompt_rows, int G, int V, SampleParams sp, hipStream_t st);
hipError_t g_score_rows(const float* logits, int n_rows, int row_offset, int V, const int* row_seq_pos,
                        const int* n_rows_dev, const int32_t* tokens, int T, float* out_logprobs, hipStream_t st);
hipError_t g_advantages(const float* rewards, int S, int G, float* out, hipStream_t st);
// y = a x
hipError_t g_scale_f32(const float* x, float a, float* y, size_t n, hipStream_t st);
// x[m][n] += bias[n]
hipError_t g_add_row_bias(float* x, const float* bias, int M, int N, hipStream_t st);
// out[s] = len[s] if the sequence has stopped (len > 0), else max_new
hipError_t g_lengths_out(const int* len, int S, int max_new, int32_t* out, hipStream_t st);
// slot_seq[0 .. n_slots): the running sequences (len[s] == 0) in ascending order, then ended ones in ascending
// order as fill (n_slots <= S; the caller makes sure that at most n_slots sequences are running).
hipError_t g_compact_slots(const int* len, int S, int n_slots, int* slot_seq, hipStream_t st);
hipError_t g_assemble(const int32_t* local_tokens, const float* local_rewards, int n_local_pool, const int32_t* ext_tokens,
                      const float* ext_rewards, int n_ext_pool, int G, int T, int n_local, int n_ext, uint32_t seed_lo,
                      uint32_t seed_hi, int32_t* out_tokens, float* out_rewards, int* out_source, int* out_counts,
                      void* workspace, hipStream_t st);
size_t g_surrogate_workspace_bytes();
hipError_t g_surrogate_loss(const float* logp_new, const float* logp_old, const uint8_t* mask, const float* adv, int S, int T,
                            float eps_low, float eps_high, float* out_loss, float* out_dlogp, void* workspace,
                            hipStream_t st);
hipError_t g_page_table(int* pt, int n_seq, int pages_per_seq, int G, int full_prompt_pages, int n_prompts,
                        hipStream_t st);
hipError_t g_copy_partial_page(int dtype, KVCache kv, int n_prompts, int G, int page_idx, hipStream_t st);
// the same with one prompt length per prompt (device): page lens[p] / 16 of prompt p, if partly filled
hipError_t g_copy_partial_page_ragged(int dtype, KVCache kv, int n_prompts, int G, const int* lens, hipStream_t st);
// page table for prompts of different lengths: fp_max shared page slots per prompt, `own` pages per sequence
hipError_t g_page_table_ragged(int* pt, int n_seq, int pages_per_seq, int G, int fp_max, int own, int n_prompts,
                               const int* lens, hipStream_t st);
hipError_t g_fill_i32(int* p, int v, size_t n, hipStream_t st);
// counter += number of IEEE-half elements equal to +-65504 (the value the float -> half conversion clamps to) among the
// rows < rows_valid of buf; x32 != 0: buf is in 32-row fragment order (blocks of 32 rows x 16 k), else row-major
hipError_t g_count_half_at_limit(const void* buf, int rows_valid, int row_len, int x32, unsigned long long* counter,
                                 hipStream_t st);
hipError_t g_fill_f32(float* p, float v, size_t n, hipStream_t st);
hipError_t g_incr(int* p, hipStream_t st);
hipError_t g_masked_rows(const uint8_t* mask, int T, int s0, int ns, int* rows /*[ns*T,2]*/, int* src_rows /*[ns*T]*/,
                         int* count, hipStream_t st);
hipError_t g_rows_from_positions(const int* positions, int n, int T, int* src_rows, hipStream_t st);
hipError_t g_last_rows(int* rows, int P, int Lp, hipStream_t st);
hipError_t g_gumbel(uint32_t seed_lo, uint32_t seed_hi, uint32_t seq, uint32_t step, uint32_t v0, int n, float* out,
                    hipStream_t st);

}  // namespace sapo

// =======================================================================================
// MFMA (bf16) kernels: weights live in "fragment order" so that a wave's operand load for one
// 32x32x16 MFMA step is one contiguous 1 KiB read:
//   Wp[((tile * (K/16) + ks) * 64 + lane) * 8 + e] = W[tile*32 + lane%32][ks*16 + (lane/32)*8 + e]
// =======================================================================================
namespace sapo {

struct BigEpi {
  int mode;            // see enum below
  float* out_f32;      // STORE_F32 / ADD_F32: [M, ldc]
  int ldc;
  f16* out_act;        // SWIGLU: act, X32 order over F = N / 2
  // RMSNorm folded around the GEMM (a row's scale commutes with the contraction).  Consumer side: the
  // token operand holds x * gain without the row scale; the accumulators are multiplied by
  // rsqrt(sum of the row's ssq parts / norm_dim + eps) before the epilogue proper.
  const float* bias = nullptr;     // STORE_F32, optional: [N] added after the row scale
  // Split-K (STORE_F32, M <= 256 only): split z of `splits` (a multiple of 8) covers about 1/splits of K and stores
  // to out_f32 + z * split_stride.
  int splits = 1;
  size_t split_stride = 0;
  bool decode = false;   // accounting only: a launch of the decode step (weight-streaming-bound)
  const float* ssq_in = nullptr;   // [M, ssq_parts rounded up to a multiple of 4]; at most 16 parts
  int ssq_parts = 0;
  float norm_dim = 0.f, eps = 0.f;
  // Producer side (ADD_F32 only): the updated residual row, times gain_next, goes out as half in X32
  // order (the next GEMM's operand), and its sum of squares in N / 128 parts per row.
  const float* gain_next = nullptr;   // [N]
  f16* xn_out = nullptr;
  float* ssq_out = nullptr;           // [M, N / 128 rounded up to a multiple of 4]
};
enum { BIG_STORE_F32 = 0, BIG_ADD_F32 = 1, BIG_SWIGLU = 2 };

// QKV projection with rotary embedding + KV append in the epilogue (head_dim 64 or 128)
struct QkvEpi {
  const float* ssq_in = nullptr;   // row scale of the folded norm, as in BigEpi
  int ssq_parts = 0;
  float norm_dim = 0.f, eps = 0.f;
  const float* bias = nullptr;     // [N] optional
  const float2* rope = nullptr;    // [max_seq][hd / 2] (cos, sin)
  RowMap rm;
  KVCache kv;
  f16* q_out = nullptr;            // [M, Hq hd] rotated queries, half
  int n_q_heads = 0;
};
hipError_t m_gemm_qkv_rope(const void* Xp, const void* Wp, int M, int N, int K, const QkvEpi& epi, hipStream_t st);

constexpr int kPackRangeSlots = 512;   // pairs of range counters behind m_pack_weight's `range`
hipError_t m_pack_weight(const void* src, int n_rows, int K, void* dst, int dst_tile0, int dst_tile_stride, unsigned* range,
                         hipStream_t st);
// Xp: tokens in X32 fragment order (rows padded to a multiple of 32); Wp: weights in W32 order
hipError_t m_gemm_big(const void* Xp, const void* Wp, int M, int N, int K, BigEpi epi, hipStream_t st);
hipError_t m_rmsnorm_x32(const float* h, const float* gain, float eps, void* out, int M, int d, const int* row_index,
                         hipStream_t st);
hipError_t m_lmhead_score(const void* Xp, const void* Wp, int max_rows, const int* n_rows_dev, int V, int K,
                          const int* row_seq_pos, const int32_t* tokens, int T, float* partials, float* out_logprobs,
                          hipStream_t st);
size_t m_lmhead_score_partial_floats(int max_rows, int V);
// Fused LM head + sampler for any number of sequences and any K: Xp = final-normed rows in X32 order.
// partials: [m_lmhead_sample_big_groups(V)][n_rows][5].
int m_lmhead_sample_big_groups(int V);
hipError_t m_lmhead_sample_big(const void* Xp, const void* Wp, int n_rows, int V, int K, SampleParams sp, float* partials,
                               hipStream_t st);
// causal GQA attention over rows laid out [n_seq, rm.T] (block mode), K/V from the paged cache;
// q row-major, out in X32 order
hipError_t m_flash_attention(const void* q, RowMap rm, KVCache kv, void* out, int n_seq, int n_q_heads, hipStream_t st);

// decode kernels (kernels_decode.hip) -------------------------------------------------------
enum { SKM_STORE = 0, SKM_RESID = 1, SKM_SWIGLU = 2 };
struct SkinnyArgs {
  const uint4* Wp;        // weights, W16 fragment order [N/16][K/32][64]
  const uint4* Xp;        // tokens, X16 order [blocks][K/32][4][64]
  int N, K, n_rows;
  int s_pad;              // 64 * number of token blocks: row stride of the ssq arrays
  // STORE, SWIGLU: accumulators are scaled by rsqrt(sum_p ssq_in[p][tok] / norm_dim + eps)
  const float* ssq_in;    // [ssq_parts][s_pad]
  int ssq_parts;
  int norm_dim;
  float eps;
  float* out_f32;         // STORE: [n_rows, ldc]
  int ldc;
  const float* bias;      // STORE, optional: [N] added after the scale
  float* h;               // RESID: residual stream [n_rows, N], updated in place
  const float* gain_next; // RESID: gain of the norm that reads the updated residual [N]
  uint4* xp_out;          // RESID: half(h * gain_next), X16 order over K' = N; SWIGLU: act, X16 order over K' = N / 2
  float* ssq_out;         // RESID: [N/16][s_pad] sums of h^2 over each 16-feature tile
};
hipError_t d_pack_weight16(const void* src, int n_rows, int K, void* dst, int dst_tile0, int dst_tile_stride,
                           hipStream_t st);
hipError_t d_gemm_skinny(const SkinnyArgs& a, int mode, hipStream_t st);
hipError_t d_pack_rows_x16(const float* h, const float* gain, int M, int d, void* xp, float* ssq, hipStream_t st);
// h += sum_z partial[z] (z < splits, each [M, d], split_stride floats apart), then xp and ssq[(d + 1023) / 1024][s_pad]
hipError_t d_resid_finish_x16(const float* partial, int splits, size_t split_stride, float* h, const float* gain, int M, int d,
                              int s_pad, void* xp, float* ssq, hipStream_t st);
// Row m <- the embedding of the token that sequence m (slot_seq[m] when slot_seq is given) emitted at step *step - 1
hipError_t d_embed_x16(const int32_t* tokens, int tok_stride, const int* step, const void* embed, int M, int d,
                       const float* gain, float* h, void* xp, float* ssq, const int* slot_seq, hipStream_t st);
bool d_lmhead_sample_supported(int K, int n_rows);
size_t d_lmhead_sample_partial_floats();
// Fused LM head + sampler for at most 64 sequences, followed by the merge that writes token and
// log-prob of the step and gathers the token's embedding row for the next step (h, X16 row with
// gain_first, one ssq part).
hipError_t d_lmhead_sample(const void* Wp, const void* Xp, int K, int V, const float* ssq, int ssq_parts, int s_pad,
                           float eps, int n_rows, SampleParams sp, float* partials, const void* embed,
                           const float* gain_first, float* h, void* xp_first, float* ssq_first, hipStream_t st);
// Merge of sampler partials [n_parts][row_stride][5] of n_rows sequences: token + log-prob of the step,
// then the embedding gather for the next step.
hipError_t d_lmhead_merge_embed(const float* partials, int n_parts, int row_stride, int n_rows, SampleParams sp,
                                const void* embed, int d, const float* gain_first, float* h, void* xp_first,
                                float* ssq_first, hipStream_t st);
// Decode attention with the prompt's pages read once per group of siblings (rows = P prompts x G siblings in order,
// every sequence at the same position, the siblings' page tables pointing at the same pages for the first
// 2 * prefix_pairs pages).  The launch then holds two kinds of workgroups: block ids 0 .. n_prefix - 1, one per
// (prompt, KV head), cover those pages for all siblings' query heads at once and leave per (row, query head) the
// unnormalised partial result (running max, sum, weighted values) in `pre`; the others, one per (row, KV head), cover
// the row's remaining tokens and fold the partial result in once the prefix workgroup's flag shows this launch's number.
struct ShareArgs {
  int G = 0;                  // siblings per prompt
  int prefix_pairs = 0;       // shared page pairs (32 tokens each); 0: no sharing
  int n_prefix = 0;           // P x KV heads
  float* pre = nullptr;       // [rows][n_q_heads][head_dim + 4]: m, l, -, -, o[head_dim]
  unsigned* flags = nullptr;  // [n_prefix], zero when the call begins; launch number = step * n_layers + layer + 1
  unsigned* fault = nullptr;  // set when a wait gave up
  int layer = 0, n_layers = 1;
  unsigned spin_ticks = 20000000u;   // bound of the wait in ticks of the 100 MHz wall clock
};
constexpr int kSharePrefixMaxColumns = 64;   // G x (query heads per KV head) the prefix workgroups can take
hipError_t d_decode_attention(const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* out_x16, int S,
                              int n_q_heads, const ShareArgs* share, hipStream_t st);

// One decode step's layers as one persistent kernel (decode_persist.hip), up to 64 rows ----------------------
// Exchange counters between the resident workgroups; zeroed once at the start of a rollout call, then only growing
// (launch n since then starts from n x the arrivals of one launch).
struct PersistCtl {
  unsigned global;         // arrival groups that have completed a phase, summed over phases and launches
  unsigned pad0[63];
  unsigned group[8][64];   // one counter per arrival group, each in a 256-byte line of its own
  unsigned fault;          // set when a wait ran into its time limit: the step's results are not valid
  unsigned pad1[63];
  unsigned launches;       // launches of the persistent kernel since the counters were zeroed (moved on by the last
  unsigned pad2[63];       // workgroup to report the last phase of a launch)
};
struct PersistLayer {      // device table, one entry per layer (weights in W16 fragment order)
  const uint4 *wqkv, *wo, *wgu, *wdown;
  const float *bqkv, *ffn_norm, *gain_after;   // gain_after: the next layer's attention norm, or the final norm
};
struct PersistArgs {
  int n_layers, S, s_pad, d, q_dim, kv_dim, F, n_q_heads;
  float eps;
  const PersistLayer* layers;
  float* h;                // [S, d] residual stream
  float* qkv;              // [S, q + 2 kv]
  uint4* attn;             // X16 [s_pad, q]
  uint4* xa;               // X16 [s_pad, d]: QKV projection's operand (in: from the sampler's merge; out: for the LM head)
  uint4* xb;               // X16 [s_pad, d]: gate / up projection's operand
  uint4* act;              // X16 [s_pad, F]
  float* ssq_a;            // [d / 16][s_pad]; one part on entry
  float* ssq_b;            // [d / 16][s_pad]
  const float2* rope;
  RowMap rm;               // decode mode
  KVCache kv0;             // layer 0's cache
  size_t kv_layer_stride;  // bytes from a layer's K (V) pool to the next layer's
  PersistCtl* ctl;
  int v_qkv, v_o, v_gu, v_down;   // blocking of each GEMM phase (set by the launcher)
  unsigned spin_ticks;            // limit of one wait in ticks of the 100 MHz wall clock (set by the launcher)
};
size_t d_decode_layers_ctl_bytes();
bool d_decode_layers_supported(int S, int d, int q_dim, int kv_dim, int F, int head_dim, int n_kv_heads);
// kernel attributes and the residency check, once per process and outside any stream capture; the launch needs it
hipError_t d_decode_layers_prepare();
hipError_t d_decode_layers(PersistArgs args, int head_dim, hipStream_t st);

hipError_t g_gather_last_rows(const float* h, float* out, int S, int G, int Lp, int d, hipStream_t st);
// with per-prompt lengths (device): row p * Lp + lens[p] - 1
hipError_t g_gather_last_rows_ragged(const float* h, float* out, int S, int G, int Lp, const int* lens, int d,
                                     hipStream_t st);

}  // namespace sapo
