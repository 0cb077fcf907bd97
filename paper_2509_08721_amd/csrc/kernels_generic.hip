// Shape-generic kernels: any model shape, fp32 or bf16 storage, plain ALU arithmetic.
// They run the fp32 configuration and every step that has no tile-aligned MFMA kernel.
#include "common.h"
#include "surrogate.h"
#include "train.h"
#include <mutex>

namespace sapo {

#define SAPO_DISPATCH_T(dtype, ...)                                   \
  do {                                                                \
    if ((dtype) == SAPO_DTYPE_F32) { typedef float T; __VA_ARGS__; }  \
    else { typedef bf16 T; __VA_ARGS__; }                             \
  } while (0)

// ---------------------------------------------------------------------------------------
// small utilities
// ---------------------------------------------------------------------------------------
__global__ void k_fill_i32(int* p, int v, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void k_fill_f32(float* p, float v, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void k_incr(int* p) { if (threadIdx.x == 0) *p += 1; }

// 8 halfs per thread; a wave adds its count with one atomic
__global__ void k_count_half_at_limit(const uint4* __restrict__ buf, size_t n_chunks, int rows_valid, int row_len, int x32,
                                      unsigned long long* __restrict__ counter) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  unsigned hits = 0;
  if (i < n_chunks) {
    // row of chunk i: row-major rows hold row_len / 8 chunks; fragment order holds 64 chunks per (32 rows x 16 k) block
    const size_t row = x32 ? (i / ((size_t)64 * (row_len >> 4))) * 32 + (i & 31) : i / (size_t)(row_len >> 3);
    if (row < (size_t)rows_valid) {
      const uint4 v = buf[i];
      const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        hits += ((w[e] & 0x7fffu) == 0x7bffu);
        hits += (((w[e] >> 16) & 0x7fffu) == 0x7bffu);
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off, 64);
  if ((threadIdx.x & 63) == 0 && hits) atomicAdd(counter, (unsigned long long)hits);
}
hipError_t g_count_half_at_limit(const void* buf, int rows_valid, int row_len, int x32, unsigned long long* counter,
                                 hipStream_t st) {
  if (rows_valid <= 0 || row_len <= 0) return hipSuccess;
  if (row_len % 16 != 0) return hipErrorInvalidValue;
  const size_t rows = x32 ? ((size_t)rows_valid + 31) / 32 * 32 : (size_t)rows_valid;
  const size_t n_chunks = rows * (size_t)row_len / 8;
  return launch(KID_MISC, k_count_half_at_limit, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st, (const uint4*)buf,
                n_chunks, rows_valid, row_len, x32, counter);
}

hipError_t g_fill_i32(int* p, int v, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  return launch(KID_MISC, k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
}
hipError_t g_fill_f32(float* p, float v, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  return launch(KID_MISC, k_fill_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
}
hipError_t g_incr(int* p, hipStream_t st) {
  return launch(KID_MISC, k_incr, dim3(1), dim3(64), 0, st, p);
}

// Page table: the first `full_prompt_pages` pages of a sequence are its prompt's shared pages,
// the rest are the sequence's own.
__global__ void k_page_table(int* pt, int n_seq, int pages_per_seq, int G, int fp, int n_prompts) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_seq * pages_per_seq) return;
  int s = i / pages_per_seq, j = i % pages_per_seq;
  int own = pages_per_seq - fp;
  pt[i] = (j < fp) ? (s / G) * fp + j : n_prompts * fp + s * own + (j - fp);
}
__global__ void k_page_table_ragged(int* pt, int n_seq, int pages_per_seq, int G, int fp_max, int own, int n_prompts,
                                    const int* __restrict__ lens) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_seq * pages_per_seq) return;
  int s = i / pages_per_seq, j = i % pages_per_seq;
  int fp = lens[s / G] / kPageTokens;
  // entries past the pages the sequence can reach point at its last own page (only padding rows read them)
  pt[i] = (j < fp) ? (s / G) * fp_max + j : n_prompts * fp_max + s * own + min(j - fp, own - 1);
}
hipError_t g_page_table_ragged(int* pt, int n_seq, int pages_per_seq, int G, int fp_max, int own, int n_prompts,
                               const int* lens, hipStream_t st) {
  int n = n_seq * pages_per_seq;
  return launch(KID_MISC, k_page_table_ragged, dim3((n + 255) / 256), dim3(256), 0, st, pt, n_seq, pages_per_seq, G, fp_max,
                own, n_prompts, lens);
}
hipError_t g_page_table(int* pt, int n_seq, int pages_per_seq, int G, int fp, int n_prompts, hipStream_t st) {
  int n = n_seq * pages_per_seq;
  return launch(KID_MISC, k_page_table, dim3((n + 255) / 256), dim3(256), 0, st, pt, n_seq, pages_per_seq, G, fp, n_prompts);
}

// Copy the (partially filled) page `page_idx` of each prompt's first sibling to the other
// siblings, both K and V.
template <typename T>
__global__ void k_copy_partial_page(KVCache kv, int G, int page_idx, const int* __restrict__ lens) {
  const int p = blockIdx.x, g = blockIdx.y + 1;
  if (lens) {
    if (lens[p] % kPageTokens == 0) return;
    page_idx = lens[p] / kPageTokens;
  }
  const int src = kv.page_table[(size_t)(p * G) * kv.pages_per_seq + page_idx];
  const int dst = kv.page_table[(size_t)(p * G + g) * kv.pages_per_seq + page_idx];
  const size_t n = (size_t)kv.n_kv_heads * kPageTokens * kv.head_dim;
  T* k = (T*)kv.k; T* v = (T*)kv.v;
  for (size_t i = threadIdx.x; i < n; i += blockDim.x) {
    k[dst * n + i] = k[src * n + i];
    v[dst * n + i] = v[src * n + i];
  }
}
hipError_t g_copy_partial_page(int dtype, KVCache kv, int n_prompts, int G, int page_idx, hipStream_t st) {
  if (G <= 1) return hipSuccess;
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_MISC, k_copy_partial_page<T>, dim3(n_prompts, G - 1), dim3(256), 0, st, kv, G, page_idx,
                                    (const int*)nullptr));
  return e;
}
hipError_t g_copy_partial_page_ragged(int dtype, KVCache kv, int n_prompts, int G, const int* lens, hipStream_t st) {
  if (G <= 1) return hipSuccess;
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_MISC, k_copy_partial_page<T>, dim3(n_prompts, G - 1), dim3(256), 0, st, kv, G, 0, lens));
  return e;
}

// ---------------------------------------------------------------------------------------
// embedding gather: h[m, :] = embed[token(m), :]
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void k_embed(const int32_t* tokens, int tok_stride, const int* step, const T* embed, float* h, int d) {
  const int m = blockIdx.x;
  const int tok = step ? tokens[(size_t)m * tok_stride + (*step - 1)] : tokens[(size_t)m * tok_stride];
  const T* e = embed + (size_t)tok * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)m * d + i] = to_f32(e[i]);
}
hipError_t g_embed(int dtype, const int32_t* tokens, int tok_stride, const int* step, const void* embed, float* h,
                   int M, int d, hipStream_t st) {
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_EMBED, k_embed<T>, dim3(M), dim3(256), 0, st, tokens, tok_stride, step, (const T*)embed, h, d));
  return e;
}

// ---------------------------------------------------------------------------------------
// RMSNorm: out[i, :] = T( h[r, :] * rsqrt(mean(h[r, :]^2) + eps) * gain ),  r = row_index ? row_index[i] : i
// row_index < 0 entries (padding) produce zeros.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void k_rmsnorm(const float* h, const float* gain, float eps, T* out, int d, const int* row_index) {
  const int i = blockIdx.x;
  const int r = row_index ? row_index[i] : i;
  T* o = out + (size_t)i * d;
  if (r < 0) {
    for (int j = threadIdx.x; j < d; j += blockDim.x) o[j] = from_f32<T>(0.f);
    return;
  }
  const float* x = h + (size_t)r * d;
  float ss = 0.f;
  for (int j = threadIdx.x; j < d; j += blockDim.x) ss += x[j] * x[j];
  __shared__ float red[4];
  ss = wave_reduce_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = red[0] + red[1] + red[2] + red[3];
  const float scale = 1.0f / sqrtf(tot / (float)d + eps);
  for (int j = threadIdx.x; j < d; j += blockDim.x) o[j] = from_f32<T>(x[j] * scale * gain[j]);
}
hipError_t g_rmsnorm(int dtype, const float* h, const float* gain, float eps, void* out, int M, int d,
                     const int* row_index, hipStream_t st) {
  if (M == 0) return hipSuccess;
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_RMSNORM, k_rmsnorm<T>, dim3(M), dim3(256), 0, st, h, gain, eps, (T*)out, d, row_index));
  return e;
}

// ---------------------------------------------------------------------------------------
// GEMM  C[m, n] (+)= sum_k A[m, k] W[n, k]   (A: T [M, K], W: T [N, K], C fp32 with row stride ldc)
// 64x64 tile per 256 threads, 4x4 outputs per thread, fp32 accumulation in k order.
// ---------------------------------------------------------------------------------------
template <typename T, int EPI>
__global__ void __launch_bounds__(256) k_gemm(const T* __restrict__ A, const T* __restrict__ W, float* __restrict__ C,
                                              int M, int N, int K, int ldc) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float sa[BK][BM + 4];
  __shared__ float sw[BK][BN + 4];
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = threadIdx.x; i < BM * BK; i += 256) {
      const int r = i / BK, c = i % BK;
      const int gm = m0 + r, gn = n0 + r, gk = k0 + c;
      sa[c][r] = (gm < M && gk < K) ? to_f32(A[(size_t)gm * K + gk]) : 0.f;
      sw[c][r] = (gn < N && gk < K) ? to_f32(W[(size_t)gn * K + gk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sa[kk][ty * 4 + i]; b[i] = sw[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      float* c = C + (size_t)gm * ldc + gn;
      if (EPI == EPI_ADD_F32) *c += acc[i][j]; else *c = acc[i][j];
    }
  }
}
hipError_t g_gemm(int dtype, const void* A, const void* W, float* C, int M, int N, int K, int ldc, GemmEpi epi,
                  hipStream_t st) {
  if (M == 0 || N == 0) return hipSuccess;
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, {
    if (epi == EPI_ADD_F32) e = launch(KID_GEMM_GENERIC, k_gemm<T, EPI_ADD_F32>, grid, dim3(256), 0, st, (const T*)A, (const T*)W, C, M, N, K, ldc);
    else e = launch(KID_GEMM_GENERIC, k_gemm<T, EPI_STORE_F32>, grid, dim3(256), 0, st, (const T*)A, (const T*)W, C, M, N, K, ldc);
  });
  return e;
}

// ---------------------------------------------------------------------------------------
// Rotary positions + KV append.  qkv fp32 [M, (Hq + 2 Hkv) hd].  For head-dim pair (i, i + hd/2):
//   (x_i, x_{i+hd/2}) <- (x_i c - x_{i+hd/2} s, x_{i+hd/2} c + x_i s),  (c, s) = rope[pos][i].
// q heads go to q_out T [M, Hq hd]; k heads (rotated) and v heads go to the row's cache page.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void k_rope_append(const float* __restrict__ qkv, const float2* __restrict__ rope, RowMap rm, KVCache kv,
                              T* __restrict__ q_out, int n_q_heads) {
  const int m = blockIdx.x;
  const int hd = kv.head_dim, half = hd / 2, hkv = kv.n_kv_heads;
  const int n_heads = n_q_heads + 2 * hkv;
  int seq, pos;
  rm.get(m, seq, pos);
  const bool keep = rm.keeps_kv(m);
  const int page = kv.page_table[(size_t)seq * kv.pages_per_seq + pos / kPageTokens];
  const int slot = pos % kPageTokens;
  const float* row = qkv + (size_t)m * n_heads * hd;
  for (int idx = threadIdx.x; idx < n_heads * half; idx += blockDim.x) {
    const int head = idx / half, i = idx % half;
    const float x1 = row[head * hd + i], x2 = row[head * hd + i + half];
    if (head < n_q_heads + hkv) {
      const float2 cs = rope[(size_t)pos * half + i];
      const float r1 = x1 * cs.x - x2 * cs.y, r2 = x2 * cs.x + x1 * cs.y;
      if (head < n_q_heads) {
        q_out[((size_t)m * n_q_heads + head) * hd + i] = from_f32<T>(r1);
        q_out[((size_t)m * n_q_heads + head) * hd + i + half] = from_f32<T>(r2);
      } else if (keep) {
        const int kh = head - n_q_heads;
        T* kp = (T*)kv.k + (((size_t)page * hkv + kh) * kPageTokens + slot) * hd;
        kp[i] = from_f32<T>(r1);
        kp[i + half] = from_f32<T>(r2);
      }
    } else if (keep) {
      const int vh = head - n_q_heads - hkv;
      T* vp = (T*)kv.v + ((size_t)page * hkv + vh) * hd * kPageTokens;
      vp[(size_t)i * kPageTokens + slot] = from_f32<T>(x1);
      vp[(size_t)(i + half) * kPageTokens + slot] = from_f32<T>(x2);
    }
  }
}
hipError_t g_rope_append(int dtype, const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* q_out, int M,
                         int n_q_heads, hipStream_t st) {
  if (M == 0) return hipSuccess;
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_ROPE_APPEND, k_rope_append<T>, dim3(M), dim3(256), 0, st, qkv, rope, rm, kv, (T*)q_out, n_q_heads));
  return e;
}

hipError_t g_rope_append_f16(const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* q_out, int M,
                             int n_q_heads, hipStream_t st) {
  if (M == 0) return hipSuccess;
  return launch(KID_ROPE_APPEND, k_rope_append<f16>, dim3(M), dim3(256), 0, st, qkv, rope, rm, kv, (f16*)q_out, n_q_heads);
}

// ---------------------------------------------------------------------------------------
// Causal grouped-query attention over the paged cache, one wave per (row, query head).
// Scores of the row's context are kept in LDS: pass 1 scores + max, pass 2 exp + sum, pass 3 PV.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_attention(const T* __restrict__ q, RowMap rm, KVCache kv, T* __restrict__ out,
                                                   int M, int n_q_heads, int max_ctx) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int hd = kv.head_dim, hkv = kv.n_kv_heads;
  const long item = (long)blockIdx.x * 4 + wave;
  if (item >= (long)M * n_q_heads) return;           // whole wave exits together; no block barriers below
  const int m = (int)(item / n_q_heads), h = (int)(item % n_q_heads);
  const int kvh = h / (n_q_heads / hkv);
  int seq, pos;
  rm.get(m, seq, pos);
  const int ctx = pos + 1;
  float* sc = smem + (size_t)wave * (max_ctx + hd);
  float* qs = sc + max_ctx;
  const T* qrow = q + ((size_t)m * n_q_heads + h) * hd;
  for (int i = lane; i < hd; i += 64) qs[i] = to_f32(qrow[i]);
  __builtin_amdgcn_wave_barrier();
  const int* pt = kv.page_table + (size_t)seq * kv.pages_per_seq;
  const float scale = 1.0f / sqrtf((float)hd);
  float mx = -INFINITY;
  for (int n = lane; n < ctx; n += 64) {
    const T* kp = (const T*)kv.k + (((size_t)pt[n / kPageTokens] * hkv + kvh) * kPageTokens + n % kPageTokens) * hd;
    float acc = 0.f;
    for (int i = 0; i < hd; ++i) acc = fmaf(qs[i], to_f32(kp[i]), acc);
    acc *= scale;
    sc[n] = acc;
    mx = fmaxf(mx, acc);
  }
  mx = wave_reduce_max(mx);
  float sum = 0.f;
  for (int n = lane; n < ctx; n += 64) {
    const float p = expf(sc[n] - mx);
    sc[n] = p;
    sum += p;
  }
  sum = wave_reduce_sum(sum);
  __builtin_amdgcn_wave_barrier();
  const float inv = 1.0f / sum;
  for (int i = lane; i < hd; i += 64) {
    float acc = 0.f;
    for (int n = 0; n < ctx; ++n) {
      const T* vp = (const T*)kv.v + ((size_t)pt[n / kPageTokens] * hkv + kvh) * hd * kPageTokens;
      acc = fmaf(sc[n], to_f32(vp[(size_t)i * kPageTokens + n % kPageTokens]), acc);
    }
    out[((size_t)m * n_q_heads + h) * hd + i] = from_f32<T>(acc * inv);
  }
}
hipError_t g_attention(int dtype, const void* q, RowMap rm, KVCache kv, void* out, int M, int n_q_heads, int max_ctx,
                       hipStream_t st) {
  if (M == 0) return hipSuccess;
  const long items = (long)M * n_q_heads;
  const size_t smem = (size_t)4 * (max_ctx + kv.head_dim) * sizeof(float);
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_ATTN_GENERIC, k_attention<T>, dim3((unsigned)((items + 3) / 4)), dim3(256), smem, st, (const T*)q, rm, kv, (T*)out,
                                                                                           M, n_q_heads, max_ctx));
  return e;
}

// ---------------------------------------------------------------------------------------
// SwiGLU: act[m, j] = T( silu(gu[m, j]) * gu[m, F + j] ),  silu(x) = x / (1 + exp(-x))
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void k_swiglu(const float* __restrict__ gu, T* __restrict__ act, int M, int F) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)M * F) return;
  const size_t m = i / F, j = i % F;
  const float g = gu[m * 2 * F + j], u = gu[m * 2 * F + F + j];
  act[i] = from_f32<T>(g / (1.0f + expf(-g)) * u);
}
hipError_t g_swiglu(int dtype, const float* gu, void* act, int M, int F, hipStream_t st) {
  const size_t n = (size_t)M * F;
  if (n == 0) return hipSuccess;
  hipError_t e = hipSuccess;
  SAPO_DISPATCH_T(dtype, e = launch(KID_SWIGLU, k_swiglu<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, gu, (T*)act, M, F));
  return e;
}

// ---------------------------------------------------------------------------------------
// Row-wise LM-head reductions on materialised fp32 logits.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void block_merge_lse(LseAcc& a, float* sm_m, float* sm_l) {
  // all 256 threads: reduce (m, l) pairs; result valid in every thread
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a.merge(__shfl_xor(a.m, o, 64), __shfl_xor(a.l, o, 64));
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sm_m[wave] = a.m; sm_l[wave] = a.l; }
  __syncthreads();
  LseAcc r; r.m = sm_m[0]; r.l = sm_l[0];
  for (int w = 1; w < 4; ++w) r.merge(sm_m[w], sm_l[w]);
  a = r;
}

// Sample one token for sequence s = row * G + sibling from logits[row, :].
__global__ void __launch_bounds__(256) k_sample_rows(const float* __restrict__ logits, int G, int V, SampleParams sp) {
  resolve_sample_params(sp);
  const int row = blockIdx.x / G, s = blockIdx.x;   // s = row * G + sibling
  const float* z = logits + (size_t)row * V;
  const int step = *sp.step;
  LseAcc lse; lse.init();
  BestAcc best; best.init();
  const int nblk = (V + 3) / 4;
  for (int b = threadIdx.x; b < nblk; b += 256) {
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (sp.temperature != 0.f) gumbel4(sp.seed_lo, sp.seed_hi, (uint32_t)s, (uint32_t)step, (uint32_t)b, g);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int v = 4 * b + j;
      if (v >= V) break;
      const float zv = z[v];
      lse.add(zv);
      const float y = (sp.temperature != 0.f) ? zv / sp.temperature + g[j] : zv;
      best.add(y, zv, v);
    }
  }
  __shared__ float sm_m[4], sm_l[4], sm_y[4], sm_z[4];
  __shared__ int sm_id[4];
  block_merge_lse(lse, sm_m, sm_l);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) best.add(__shfl_xor(best.y, o, 64), __shfl_xor(best.z, o, 64), __shfl_xor(best.id, o, 64));
  if ((threadIdx.x & 63) == 0) { sm_y[threadIdx.x >> 6] = best.y; sm_z[threadIdx.x >> 6] = best.z; sm_id[threadIdx.x >> 6] = best.id; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) best.add(sm_y[w], sm_z[w], sm_id[w]);
    emit_token(sp, s, step, best.id, best.z - (lse.m + logf(lse.l)));
  }
}
hipError_t g_sample_rows(const float* logits, int n_rows, int G, int V, SampleParams sp, hipStream_t st) {
  return launch(KID_SAMPLE_ROWS, k_sample_rows, dim3(n_rows * G), dim3(256), 0, st, logits, G, V, sp);
}

// log-prob of the teacher-forced token: row i holds the logits after position (s, t-1) where
// (s, t) = row_seq_pos[i]; writes out[s, t] = z[tokens[s, t]] - logsumexp(z).
__global__ void __launch_bounds__(256) k_score_rows(const float* __restrict__ logits, int row_offset, int V,
                                                    const int* row_seq_pos, const int* n_rows_dev,
                                                    const int32_t* tokens, int T, float* out_logprobs) {
  const int i = row_offset + blockIdx.x;
  if (i >= *n_rows_dev) return;
  const float* z = logits + (size_t)blockIdx.x * V;
  LseAcc lse; lse.init();
  for (int v = threadIdx.x; v < V; v += 256) lse.add(z[v]);
  __shared__ float sm_m[4], sm_l[4];
  block_merge_lse(lse, sm_m, sm_l);
  if (threadIdx.x == 0) {
    const int s = row_seq_pos[2 * i], t = row_seq_pos[2 * i + 1];
    const int tok = tokens[(size_t)s * T + t];
    out_logprobs[(size_t)s * T + t] = z[tok] - (lse.m + logf(lse.l));
  }
}
hipError_t g_score_rows(const float* logits, int n_rows, int row_offset, int V, const int* row_seq_pos,
                        const int* n_rows_dev, const int32_t* tokens, int T, float* out_logprobs, hipStream_t st) {
  if (n_rows == 0) return hipSuccess;
  return launch(KID_SCORE_ROWS, k_score_rows, dim3(n_rows), dim3(256), 0, st, logits, row_offset, V, row_seq_pos, n_rows_dev, tokens, T, out_logprobs);
}

// ---------------------------------------------------------------------------------------
// Group-relative advantages, one thread per group, fp64.
// ---------------------------------------------------------------------------------------
__global__ void k_advantages(const float* __restrict__ r, int n_groups, int G, float* __restrict__ out) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  const float* rg = r + (size_t)g * G;
  bool all_equal = true;
  double sum = 0.0;
  for (int i = 0; i < G; ++i) { sum += (double)rg[i]; all_equal = all_equal && (rg[i] == rg[0]); }
  if (all_equal) {
    for (int i = 0; i < G; ++i) out[(size_t)g * G + i] = 0.f;
    return;
  }
  const double mu = sum / G;
  double var = 0.0;
  for (int i = 0; i < G; ++i) { const double dlt = (double)rg[i] - mu; var += dlt * dlt; }
  const double sd = sqrt(var / G);
  for (int i = 0; i < G; ++i) out[(size_t)g * G + i] = (float)(((double)rg[i] - mu) / (sd + 1e-6));
}
__global__ void k_scale_f32(const float* __restrict__ x, float a, float* __restrict__ y, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = x[i] * a;
}
hipError_t g_scale_f32(const float* x, float a, float* y, size_t n, hipStream_t st) {
  return launch(KID_MISC, k_scale_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, a, y, n);
}
__global__ void k_add_row_bias(float* __restrict__ x, const float* __restrict__ bias, size_t total, int N) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) x[i] += bias[i % N];
}
hipError_t g_add_row_bias(float* x, const float* bias, int M, int N, hipStream_t st) {
  const size_t total = (size_t)M * N;
  return launch(KID_MISC, k_add_row_bias, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, x, bias, total, N);
}
__global__ void k_lengths_out(const int* __restrict__ len, int S, int max_new, int32_t* __restrict__ out) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s < S) out[s] = len[s] > 0 ? len[s] : max_new;
}
hipError_t g_lengths_out(const int* len, int S, int max_new, int32_t* out, hipStream_t st) {
  return launch(KID_MISC, k_lengths_out, dim3((S + 255) / 256), dim3(256), 0, st, len, S, max_new, out);
}
// One workgroup: thread i owns the sequences [i c, (i + 1) c), c = ceil(S / 256); an exclusive scan of the
// per-thread counts of running and of ended sequences gives every sequence its place.
__global__ void __launch_bounds__(256) k_compact_slots(const int* __restrict__ len, int S, int n_slots, int* __restrict__ slot_seq) {
  __shared__ int run_before[257], end_before[257];
  const int c = (S + 255) / 256, s0 = min(S, (int)threadIdx.x * c), s1 = min(S, s0 + c);
  int n_run = 0;
  for (int s = s0; s < s1; ++s) n_run += (len[s] == 0);
  run_before[threadIdx.x + 1] = n_run;
  end_before[threadIdx.x + 1] = (s1 - s0) - n_run;
  __syncthreads();
  if (threadIdx.x == 0) {
    run_before[0] = end_before[0] = 0;
    for (int i = 1; i <= 256; ++i) { run_before[i] += run_before[i - 1]; end_before[i] += end_before[i - 1]; }
  }
  __syncthreads();
  const int total_run = run_before[256];
  int r = run_before[threadIdx.x], e = total_run + end_before[threadIdx.x];
  for (int s = s0; s < s1; ++s) {
    const int slot = (len[s] == 0) ? r++ : e++;
    if (slot < n_slots) slot_seq[slot] = s;
  }
}
hipError_t g_compact_slots(const int* len, int S, int n_slots, int* slot_seq, hipStream_t st) {
  if (n_slots > S) return hipErrorInvalidValue;
  return launch(KID_MISC, k_compact_slots, dim3(1), dim3(256), 0, st, len, S, n_slots, slot_seq);
}
hipError_t g_advantages(const float* rewards, int S, int G, float* out, hipStream_t st) {
  const int ng = S / G;
  return launch(KID_MISC, k_advantages, dim3((ng + 63) / 64), dim3(64), 0, st, rewards, ng, G, out);
}

// ---------------------------------------------------------------------------------------
// Clipped surrogate of the local GRPO update (Sec. 4.2: no KL term, asymmetric clip).
// Pass 1: every block walks a contiguous slice of the [S, T] tokens and leaves (sum of
// min(rho A, clip(rho) A), number of masked tokens) in its slot; pass 2: one block adds the
// slots in index order (fp64) and writes loss and count; pass 3: the gradient, which needs
// the count.  rho and the branch decision are fp32; no atomics, so the result is reproducible.
// ---------------------------------------------------------------------------------------
constexpr int kLossBlocks = 256;
struct LossPartial { double sum; long long count; };

__global__ void __launch_bounds__(256) k_surrogate_partial(const float* __restrict__ logp_new, const float* __restrict__ logp_old,
                                                           const uint8_t* __restrict__ mask, const float* __restrict__ adv,
                                                           int T, size_t n, float eps_low, float eps_high,
                                                           LossPartial* __restrict__ part) {
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t i0 = (size_t)blockIdx.x * per, i1 = (i0 + per < n) ? i0 + per : n;
  double sum = 0.0;
  long long cnt = 0;
  for (size_t i = i0 + threadIdx.x; i < i1; i += 256) {
    if (!mask[i]) continue;
    float rho; bool act;
    sum += (double)surrogate_term(logp_new[i], logp_old[i], adv[i / T], eps_low, eps_high, rho, act);
    ++cnt;
  }
  __shared__ double s_sum[256];
  __shared__ long long s_cnt[256];
  s_sum[threadIdx.x] = sum; s_cnt[threadIdx.x] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {   // thread order: the same sum whatever the hardware does
    double t = 0.0; long long c = 0;
    for (int j = 0; j < 256; ++j) { t += s_sum[j]; c += s_cnt[j]; }
    part[blockIdx.x].sum = t; part[blockIdx.x].count = c;
  }
}
__global__ void k_surrogate_finish(LossPartial* __restrict__ part, int n_part, float* __restrict__ out_loss) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double t = 0.0; long long c = 0;
  for (int j = 0; j < n_part; ++j) { t += part[j].sum; c += part[j].count; }
  part[n_part].sum = t; part[n_part].count = c;   // slot n_part: the totals, read by the gradient pass
  out_loss[0] = c > 0 ? (float)(-t / (double)c) : 0.f;
}
__global__ void __launch_bounds__(256) k_surrogate_grad(const float* __restrict__ logp_new, const float* __restrict__ logp_old,
                                                        const uint8_t* __restrict__ mask, const float* __restrict__ adv,
                                                        int T, size_t n, float eps_low, float eps_high,
                                                        const LossPartial* __restrict__ total, float* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float g = 0.f;
  if (mask[i]) {
    const float a = adv[i / T];
    float rho; bool act;
    surrogate_term(logp_new[i], logp_old[i], a, eps_low, eps_high, rho, act);
    g = surrogate_dlogp(a, rho, act, total->count);
  }
  out[i] = g;
}
size_t g_surrogate_workspace_bytes() { return (kLossBlocks + 1) * sizeof(LossPartial); }
hipError_t g_surrogate_loss(const float* logp_new, const float* logp_old, const uint8_t* mask, const float* adv, int S, int T,
                            float eps_low, float eps_high, float* out_loss, float* out_dlogp, void* workspace,
                            hipStream_t st) {
  const size_t n = (size_t)S * T;
  LossPartial* part = (LossPartial*)workspace;
  hipError_t e = launch(KID_MISC, k_surrogate_partial, dim3(kLossBlocks), dim3(256), 0, st, logp_new, logp_old, mask, adv, T,
                        n, eps_low, eps_high, part);
  if (e != hipSuccess) return e;
  e = launch(KID_MISC, k_surrogate_finish, dim3(1), dim3(64), 0, st, part, kLossBlocks, out_loss);
  if (e != hipSuccess || !out_dlogp) return e;
  return launch(KID_MISC, k_surrogate_grad, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, logp_new, logp_old, mask,
                adv, T, n, eps_low, eps_high, (const LossPartial*)(part + kLossBlocks), out_dlogp);
}

// ---------------------------------------------------------------------------------------
// The same three passes for callers that cannot allocate (code under graph capture, serving loops, harnesses that
// forbid hipMalloc): the block partials and the totals live in a file-scope device array instead of a workspace.
// Every device holds its own copy of the array; its address is looked up once per device, with that device
// current, and kept.  All 256 partial slots and the totals slot are overwritten by every call before they are
// read, so nothing has to be cleared between calls; two calls that overlap on one device share the array and race.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[(kLossBlocks + 1) * sizeof(LossPartial)];   // 4112 bytes per device

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call on that device).
static hipError_t scratch_address(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace sapo

extern "C" int sapo_clipped_surrogate_noalloc(const float* logp_new, const float* logp_old, const uint8_t* completion_mask,
                                              const float* advantages, int S, int T, float eps_low, float eps_high,
                                              float* out_loss, float* out_dlogp, void* stream) {
  using namespace sapo;
  if (S <= 0 || T <= 0) return set_error(SAPO_EINVAL, "S and T must be positive");
  if ((long)S * T > SAPO_SURROGATE_NOALLOC_MAX_TOKENS)
    return set_error(SAPO_EINVAL, "S * T = %ld exceeds the maximum of %ld tokens of sapo_clipped_surrogate_noalloc",
                     (long)S * T, (long)SAPO_SURROGATE_NOALLOC_MAX_TOKENS);
  if (!logp_new || !logp_old || !completion_mask || !advantages || !out_loss) return set_error(SAPO_EINVAL, "NULL buffer");
  if (!(eps_low >= 0.f && eps_low < 1.f && eps_high >= 0.f)) return set_error(SAPO_EINVAL, "clip bounds out of range");
  void* ptr = nullptr;
  hipError_t e = scratch_address(&ptr);
  if (e != hipSuccess) return set_error(SAPO_EHIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
  e = g_surrogate_loss(logp_new, logp_old, completion_mask, advantages, S, T, eps_low, eps_high, out_loss, out_dlogp, ptr,
                       (hipStream_t)stream);
  if (e != hipSuccess) return set_error(SAPO_EHIP, "launch failed: %s", hipGetErrorString(e));
  return SAPO_OK;
}

namespace sapo {

// ---------------------------------------------------------------------------------------
// Training-set assembly (Sec. 3.2; Algorithm 1 "Assemble training set").  A datapoint is one
// question's whole rollout (G sequences).  k_subset_keys gives every datapoint of a pool its random
// key (word 0 of the Philox block with counter (g, 0, 0, stream)) and its eligibility (swarm pool:
// the G rewards are not all equal, i.e. the advantage is not identically zero); k_subset_rank takes
// the `take` eligible datapoints with the smallest (key, index) and gives slot slot0 + rank to each;
// k_gather_datapoints copies the rows.  Integer work only: the result is exact.
// ---------------------------------------------------------------------------------------
__global__ void k_subset_keys(const float* __restrict__ rewards, int n_groups, int G, int filter, uint32_t seed_lo,
                              uint32_t seed_hi, uint32_t stream, uint32_t* __restrict__ keys, int* __restrict__ elig) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  keys[g] = philox4x32_10((uint32_t)g, 0u, 0u, stream, seed_lo, seed_hi).x;
  int live = 1;
  if (filter) {
    live = 0;
    const float* rg = rewards + (size_t)g * G;
    for (int i = 1; i < G; ++i) live |= (rg[i] != rg[0]);
  }
  elig[g] = live;
}
__global__ void k_subset_rank(const uint32_t* __restrict__ keys, const int* __restrict__ elig, int n_groups, int take,
                              int slot0, int src0, int* __restrict__ out_source, int* __restrict__ out_count) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups || !elig[g]) return;
  const uint32_t kg = keys[g];
  int rank = 0;
  for (int h = 0; h < n_groups; ++h) {
    const uint32_t kh = keys[h];
    rank += (elig[h] && (kh < kg || (kh == kg && h < g))) ? 1 : 0;
  }
  if (rank < take) {
    out_source[slot0 + rank] = src0 + g;
    atomicAdd(out_count, 1);   // integer count: the order of the additions does not matter
  }
}
__global__ void __launch_bounds__(256) k_gather_datapoints(const int32_t* __restrict__ local_tokens,
                                                           const float* __restrict__ local_rewards, int n_local_pool,
                                                           const int32_t* __restrict__ ext_tokens,
                                                           const float* __restrict__ ext_rewards, int G, int T,
                                                           const int* __restrict__ source, int32_t* __restrict__ out_tokens,
                                                           float* __restrict__ out_rewards) {
  const int slot = blockIdx.x, i = blockIdx.y;
  const int src = source[slot];
  int32_t* dst = out_tokens + ((size_t)slot * G + i) * T;
  if (src < 0) {
    for (int t = threadIdx.x; t < T; t += 256) dst[t] = 0;
    if (threadIdx.x == 0) out_rewards[(size_t)slot * G + i] = 0.f;
    return;
  }
  const bool loc = src < n_local_pool;
  const size_t row = (size_t)(loc ? src : src - n_local_pool) * G + i;
  const int32_t* from = (loc ? local_tokens : ext_tokens) + row * T;
  for (int t = threadIdx.x; t < T; t += 256) dst[t] = from[t];
  if (threadIdx.x == 0) out_rewards[(size_t)slot * G + i] = (loc ? local_rewards : ext_rewards)[row];
}
hipError_t g_assemble(const int32_t* local_tokens, const float* local_rewards, int n_local_pool, const int32_t* ext_tokens,
                      const float* ext_rewards, int n_ext_pool, int G, int T, int n_local, int n_ext, uint32_t seed_lo,
                      uint32_t seed_hi, int32_t* out_tokens, float* out_rewards, int* out_source, int* out_counts,
                      void* workspace, hipStream_t st) {
  const int n_slots = n_local + n_ext;
  const int n_max = n_local_pool > n_ext_pool ? n_local_pool : n_ext_pool;
  uint32_t* keys = (uint32_t*)workspace;
  int* elig = (int*)workspace + n_max;
  hipError_t e = g_fill_i32(out_counts, 0, 2, st);
  if (e != hipSuccess) return e;
  if (n_slots > 0 && (e = g_fill_i32(out_source, -1, (size_t)n_slots, st)) != hipSuccess) return e;
  struct Pool { const float* r; int n, take, slot0, src0, filter; uint32_t stream; int* count; };
  const Pool pools[2] = {{local_rewards, n_local_pool, n_local, 0, 0, 0, 2u, out_counts},
                         {ext_rewards, n_ext_pool, n_ext, n_local, n_local_pool, 1, 1u, out_counts + 1}};
  for (const Pool& p : pools) {
    if (p.n == 0 || p.take == 0) continue;
    const dim3 grid((p.n + 255) / 256);
    e = launch(KID_MISC, k_subset_keys, grid, dim3(256), 0, st, p.r, p.n, G, p.filter, seed_lo, seed_hi, p.stream, keys, elig);
    if (e != hipSuccess) return e;
    e = launch(KID_MISC, k_subset_rank, grid, dim3(256), 0, st, (const uint32_t*)keys, (const int*)elig, p.n, p.take, p.slot0,
               p.src0, out_source, p.count);
    if (e != hipSuccess) return e;
  }
  if (n_slots == 0) return hipSuccess;
  return launch(KID_MISC, k_gather_datapoints, dim3(n_slots, G), dim3(256), 0, st, local_tokens, local_rewards, n_local_pool,
                ext_tokens, ext_rewards, G, T, (const int*)out_source, out_tokens, out_rewards);
}

// ---------------------------------------------------------------------------------------
// Ordered compaction of the positions to score in sequences [s0, s0 + ns): entry i of `rows`
// is (s, t) with mask[s, t] != 0 and t >= 1, in (s, t) order; *count = number of entries.
// `src_rows[i]` = local row (s - s0) * T + t - 1 whose hidden state predicts token (s, t).
// Entries past the count are filled with (-1) in src_rows so that gathers read padding.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) k_masked_rows(const uint8_t* __restrict__ mask, int T, int s0, int ns,
                                                      int* __restrict__ rows, int* __restrict__ src_rows,
                                                      int* __restrict__ count) {
  __shared__ int wave_tot[16];
  __shared__ int base;
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  const int total = ns * T;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i0 = 0; i0 < total; i0 += 1024) {
    const int i = i0 + threadIdx.x;
    int flag = 0, s = 0, t = 0;
    if (i < total) {
      s = s0 + i / T; t = i % T;
      flag = (t >= 1 && mask[(size_t)s * T + t] != 0) ? 1 : 0;
    }
    const unsigned long long bal = __ballot(flag);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; ++w) off += wave_tot[w];
    if (flag) {
      const int o = off + before;
      rows[2 * o] = s; rows[2 * o + 1] = t;
      src_rows[o] = (s - s0) * T + t - 1;
    }
    __syncthreads();
    if (threadIdx.x == 0) { int tot = 0; for (int w = 0; w < 16; ++w) tot += wave_tot[w]; base += tot; }
    __syncthreads();
  }
  for (int i = base + threadIdx.x; i < total; i += 1024) src_rows[i] = -1;
  if (threadIdx.x == 0) *count = base;
}
hipError_t g_masked_rows(const uint8_t* mask, int T, int s0, int ns, int* rows, int* src_rows, int* count,
                         hipStream_t st) {
  return launch(KID_MISC, k_masked_rows, dim3(1), dim3(1024), 0, st, mask, T, s0, ns, rows, src_rows, count);
}

// src_rows for a list of (s, t) positions: row s * T + t (debug logits).
__global__ void k_rows_from_positions(const int* positions, int n, int T, int* src_rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) src_rows[i] = positions[2 * i] * T + positions[2 * i + 1];
}
hipError_t g_rows_from_positions(const int* positions, int n, int T, int* src_rows, hipStream_t st) {
  return launch(KID_MISC, k_rows_from_positions, dim3((n + 255) / 256), dim3(256), 0, st, positions, n, T, src_rows);
}

// rows[p] = index of the last prompt position of prompt p in a [P, Lp] block.
__global__ void k_last_rows(int* rows, int P, int Lp) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < P) rows[p] = p * Lp + Lp - 1;
}
hipError_t g_last_rows(int* rows, int P, int Lp, hipStream_t st) {
  return launch(KID_MISC, k_last_rows, dim3((P + 255) / 256), dim3(256), 0, st, rows, P, Lp);
}

// out[s, :] = h[(s / G) * Lp + Lp - 1, :]: the last prompt position's residual, once per sibling.
__global__ void k_gather_last_rows(const float* __restrict__ h, float* __restrict__ out, int G, int Lp, int d,
                                   const int* __restrict__ lens) {
  const int s = blockIdx.x;
  const float* src = h + ((size_t)(s / G) * Lp + (lens ? lens[s / G] : Lp) - 1) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) out[(size_t)s * d + i] = src[i];
}
hipError_t g_gather_last_rows(const float* h, float* out, int S, int G, int Lp, int d, hipStream_t st) {
  return launch(KID_MISC, k_gather_last_rows, dim3(S), dim3(256), 0, st, h, out, G, Lp, d, (const int*)nullptr);
}
hipError_t g_gather_last_rows_ragged(const float* h, float* out, int S, int G, int Lp, const int* lens, int d,
                                     hipStream_t st) {
  return launch(KID_MISC, k_gather_last_rows, dim3(S), dim3(256), 0, st, h, out, G, Lp, d, lens);
}

__global__ void k_gumbel(uint32_t seed_lo, uint32_t seed_hi, uint32_t seq, uint32_t step, uint32_t v0, int n, float* out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t v = v0 + (uint32_t)i;
  float g[4];
  gumbel4(seed_lo, seed_hi, seq, step, v >> 2, g);
  out[i] = g[v & 3];
}
hipError_t g_gumbel(uint32_t seed_lo, uint32_t seed_hi, uint32_t seq, uint32_t step, uint32_t v0, int n, float* out,
                    hipStream_t st) {
  if (n == 0) return hipSuccess;
  return launch(KID_MISC, k_gumbel, dim3((n + 255) / 256), dim3(256), 0, st, seed_lo, seed_hi, seq, step, v0, n, out);
}

}  // namespace sapo
