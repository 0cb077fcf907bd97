// bf16 MFMA kernels for gfx950 used when many tokens go through the layers at once (prefill and
// scoring): weight packing, the token-parallel ("big") GEMM, and the fused LM head of the scoring
// pass (log-softmax + target gather).
#include "common.h"

namespace sapo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
union Frag {
  uint4 u;
  u32x4 n;
  bf16x8 v;
};

__device__ __forceinline__ f32x16 mfma32(const Frag& a, const Frag& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(const Frag& a, const Frag& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ---------------------------------------------------------------------------------------
// weight packing: row-major [n_rows, K] -> fragment order, 32-row tiles placed at
// dst_tile0 + t * dst_tile_stride (stride 2 interleaves gate and up tiles).
// ---------------------------------------------------------------------------------------
__global__ void k_pack_weight(const bf16* __restrict__ src, int n_rows, int K, uint4* __restrict__ dst, int tile0,
                              int tile_stride) {
  const int KS = K >> 4;
  const size_t total = (size_t)(n_rows >> 5) * KS * 64;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const int ks = (int)((idx >> 6) % KS);
  const int t = (int)((idx >> 6) / KS);
  const int row = t * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
  const uint4 v = *(const uint4*)(src + (size_t)row * K + k);
  dst[((size_t)(tile0 + t * tile_stride) * KS + ks) * 64 + lane] = v;
}
hipError_t m_pack_weight(const void* src, int n_rows, int K, void* dst, int dst_tile0, int dst_tile_stride,
                         hipStream_t st) {
  const size_t total = (size_t)(n_rows / 32) * (K / 16) * 64;
  if (total == 0) return hipSuccess;
  return launch(KID_MISC, k_pack_weight, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16*)src, n_rows, K, (uint4*)dst, dst_tile0,
                                                                  dst_tile_stride);
}

// =======================================================================================
// Big GEMM:  C^T[feat, tok] = sum_k W[feat, k] X[tok, k]
// Workgroup tile 128 features x 256 tokens, 4 waves as 2 (features) x 2 (tokens); each wave owns
// 64 features x 128 tokens = 2 x 4 MFMA 32x32 tiles.  W fragments go straight from global memory
// (fragment order, 1 KiB per wave per step) into registers; X is staged through LDS in fragment
// order, 32 k per stage, double buffered.
// Accumulator layout: acc[fi][tj][4 i + j] = C^T[feat = fi*32 + (lane/32)*4 + 8 i + j][tok = tj*32 + lane%32].
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void big_mainloop(const bf16* __restrict__ X, int ldx, const uint4* __restrict__ Wp, int M,
                                             int K, int ft, int tok0, uint4* smem, f32x16 (&acc)[2][4]) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wf = wave & 1, wt = wave >> 1;
  const int KS = K >> 4, nst = KS >> 1;
  const uint4* wb0 = Wp + ((size_t)(ft * 4 + wf * 2 + 0) * KS) * 64 + lane;
  const uint4* wb1 = Wp + ((size_t)(ft * 4 + wf * 2 + 1) * KS) * 64 + lane;
  uint4 xr[4];
  Frag wc[4], wn[4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  auto load_x = [&](int st) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = i * 256 + tid, tok = c >> 2, kc = c & 3;
      const int gt = tok0 + tok;
      xr[i] = (gt < M) ? *(const uint4*)(X + (size_t)gt * ldx + st * 32 + kc * 8) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = i * 256 + tid, tok = c >> 2, kc = c & 3;
      smem[buf * 1024 + ((kc >> 1) * 8 + (tok >> 5)) * 64 + (tok & 31) + 32 * (kc & 1)] = xr[i];
    }
  };
  auto load_w = [&](int st, Frag* w) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      w[s2 * 2 + 0].u = wb0[(size_t)(st * 2 + s2) * 64];
      w[s2 * 2 + 1].u = wb1[(size_t)(st * 2 + s2) * 64];
    }
  };

  load_x(0);
  load_w(0, wc);
  store_x(0);
  __syncthreads();
  for (int st = 0; st < nst; ++st) {
    const int buf = st & 1;
    if (st + 1 < nst) {
      load_x(st + 1);
      load_w(st + 1, wn);
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      Frag xf[4];
#pragma unroll
      for (int tj = 0; tj < 4; ++tj) xf[tj].u = smem[buf * 1024 + (s2 * 8 + wt * 4 + tj) * 64 + lane];
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) acc[fi][tj] = mfma32(wc[s2 * 2 + fi], xf[tj], acc[fi][tj]);
    }
    if (st + 1 < nst) {
      store_x(buf ^ 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) wc[i] = wn[i];
    }
    __syncthreads();
  }
}

__global__ void __launch_bounds__(256) k_gemm_big(const bf16* __restrict__ X, int ldx, const uint4* __restrict__ Wp,
                                                  int M, int N, int K, BigEpi ep) {
  __shared__ uint4 smem[2048];
  const int ft = blockIdx.x, tok0 = blockIdx.y * 256;
  f32x16 acc[2][4];
  big_mainloop(X, ldx, Wp, M, K, ft, tok0, smem, acc);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wf = wave & 1, wt = wave >> 1;
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    const int tok = tok0 + wt * 128 + tj * 32 + (lane & 31);
    if (tok >= M) continue;
    if (ep.mode == BIG_SWIGLU) {
      const int F = N >> 1;
      const int f0 = (ft * 2 + wf) * 32 + (lane >> 5) * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bf16x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = (bf16)(silu_f(acc[0][tj][4 * i + j]) * acc[1][tj][4 * i + j]);
        *(bf16x4*)(ep.out_bf16 + (size_t)tok * F + f0 + 8 * i) = o;
      }
    } else {
#pragma unroll
      for (int fi = 0; fi < 2; ++fi) {
        const int f0 = ft * 128 + wf * 64 + fi * 32 + (lane >> 5) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float4* p = (float4*)(ep.out_f32 + (size_t)tok * ep.ldc + f0 + 8 * i);
          float4 v = make_float4(acc[fi][tj][4 * i], acc[fi][tj][4 * i + 1], acc[fi][tj][4 * i + 2], acc[fi][tj][4 * i + 3]);
          if (ep.mode == BIG_ADD_F32) {
            const float4 o = *p;
            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
          }
          *p = v;
        }
      }
    }
  }
}
hipError_t m_gemm_big(const void* X, int ldx, const void* Wp, int M, int N, int K, BigEpi epi, hipStream_t st) {
  if (M == 0) return hipSuccess;
  dim3 grid(N / 128, (M + 255) / 256);
  return launch(KID_GEMM_BIG, k_gemm_big, grid, dim3(256), 0, st, (const bf16*)X, ldx, (const uint4*)Wp, M, N, K, epi);
}

// ---------------------------------------------------------------------------------------
// LM head for scoring: log-softmax + target gather without materialising logits.
// grid (token tiles of 256, kScoreSplit vocabulary ranges).  Each workgroup walks its range of
// 128-feature tiles for its 256 rows keeping a running (max, sum exp) per row, and the one lane
// that sees the row's target id writes the target logit.  A second kernel merges the ranges.
// partials: [kScoreSplit][max_rows][2] then ztarget [max_rows].
// ---------------------------------------------------------------------------------------
constexpr int kScoreSplit = 8;
size_t m_lmhead_score_partial_floats(int max_rows) { return (size_t)max_rows * (2 * kScoreSplit + 1); }

__global__ void __launch_bounds__(256) k_lmhead_score(const bf16* __restrict__ X, const uint4* __restrict__ Wp,
                                                      int max_rows, const int* __restrict__ n_rows_dev, int V, int K,
                                                      const int* __restrict__ row_seq_pos,
                                                      const int32_t* __restrict__ tokens, int T,
                                                      float* __restrict__ partials) {
  __shared__ uint4 smem[2048];
  __shared__ float red_m[2][256], red_l[2][256];
  const int n_rows = *n_rows_dev;
  const int tok0 = blockIdx.x * 256;
  if (tok0 >= n_rows) return;
  const int n_ft = V / 128;
  const int per = (n_ft + kScoreSplit - 1) / kScoreSplit;
  const int ft_begin = blockIdx.y * per, ft_end = min(n_ft, ft_begin + per);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wf = wave & 1, wt = wave >> 1;
  LseAcc lse[4];
  int target[4];
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    lse[tj].init();
    const int row = tok0 + wt * 128 + tj * 32 + (lane & 31);
    target[tj] = -1;
    if (row < n_rows) target[tj] = tokens[(size_t)row_seq_pos[2 * row] * T + row_seq_pos[2 * row + 1]];
  }
  float* ztarget = partials + (size_t)max_rows * 2 * kScoreSplit;
  for (int ft = ft_begin; ft < ft_end; ++ft) {
    f32x16 acc[2][4];
    big_mainloop(X, K, Wp, n_rows, K, ft, tok0, smem, acc);
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      const int row = tok0 + wt * 128 + tj * 32 + (lane & 31);
#pragma unroll
      for (int fi = 0; fi < 2; ++fi) {
        const int f0 = ft * 128 + wf * 64 + fi * 32 + (lane >> 5) * 4;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float z = acc[fi][tj][v];
          lse[tj].add(z);
          if (f0 + 8 * (v >> 2) + (v & 3) == target[tj]) ztarget[row] = z;
        }
      }
    }
  }
  // merge the two lane halves, then the two feature waves of each token half
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    lse[tj].merge(__shfl_xor(lse[tj].m, 32, 64), __shfl_xor(lse[tj].l, 32, 64));
    if (lane < 32) {
      red_m[wf][wt * 128 + tj * 32 + lane] = lse[tj].m;
      red_l[wf][wt * 128 + tj * 32 + lane] = lse[tj].l;
    }
  }
  __syncthreads();
  const int row = tok0 + threadIdx.x;
  if (row < n_rows) {
    LseAcc a;
    a.m = red_m[0][threadIdx.x]; a.l = red_l[0][threadIdx.x];
    a.merge(red_m[1][threadIdx.x], red_l[1][threadIdx.x]);
    float* p = partials + ((size_t)blockIdx.y * max_rows + row) * 2;
    p[0] = a.m; p[1] = a.l;
  }
}

__global__ void k_lmhead_score_merge(const float* __restrict__ partials, int max_rows, const int* __restrict__ n_rows_dev,
                                     const int* __restrict__ row_seq_pos, int T, float* __restrict__ out_logprobs) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= *n_rows_dev) return;
  LseAcc a; a.init();
  for (int s = 0; s < kScoreSplit; ++s) {
    const float* p = partials + ((size_t)s * max_rows + row) * 2;
    a.merge(p[0], p[1]);
  }
  const float zt = partials[(size_t)max_rows * 2 * kScoreSplit + row];
  out_logprobs[(size_t)row_seq_pos[2 * row] * T + row_seq_pos[2 * row + 1]] = zt - (a.m + logf(a.l));
}

hipError_t m_lmhead_score(const void* X, const void* Wp, int max_rows, const int* n_rows_dev, int V, int K,
                          const int* row_seq_pos, const int32_t* tokens, int T, float* partials, float* out_logprobs,
                          hipStream_t st) {
  if (max_rows == 0) return hipSuccess;
  dim3 grid((max_rows + 255) / 256, kScoreSplit);
  const hipError_t e = launch(KID_LMHEAD_SCORE, k_lmhead_score, grid, dim3(256), 0, st, (const bf16*)X, (const uint4*)Wp, max_rows,
                              n_rows_dev, V, K, row_seq_pos, tokens, T, partials);
  if (e != hipSuccess) return e;
  return launch(KID_LMHEAD_SCORE_MERGE, k_lmhead_score_merge, dim3((max_rows + 255) / 256), dim3(256), 0, st, partials, max_rows, n_rows_dev, row_seq_pos, T,
                                                               out_logprobs);
}

// =======================================================================================
// Causal GQA attention for prefill and scoring (many positions per sequence), MFMA 16x16x32.
// grid (64-position blocks, longest first; sequences x KV heads; groups of HPW query heads).
// A wave owns 16 query positions and up to HPW query heads that share the KV head, and walks the
// keys 0 .. last query position in 32-key page pairs read straight from the paged cache into
// fragment registers: S^T = K Q^T puts one query column in each lane, so the running max / sum are
// per-lane scalars (plus two shuffles) and the probabilities a lane produces are its operand of
// O^T = V^T P^T; key rows are permuted inside a pair so that a lane's 8 probabilities are 8
// consecutive tokens, the unit the token-minor V page delivers in one 16-byte load.  No LDS, no
// block-level synchronisation; waves never exchange data.
// ---------------------------------------------------------------------------------------
template <int HD, int HPW>
__global__ void __launch_bounds__(256) k_flash_attention(const bf16* __restrict__ q, RowMap rm, KVCache kv,
                                                         bf16* __restrict__ out, int n_q_heads) {
  constexpr int KK = HD / 32, DT = HD / 16;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int qcol = lane & 15, grp = lane >> 4;
  const int T = rm.T;
  const int qb = gridDim.x - 1 - blockIdx.x;
  const int hkv = kv.n_kv_heads, rep = n_q_heads / hkv;
  const int sblk = blockIdx.y / hkv, kvh = blockIdx.y % hkv;
  const int h0 = blockIdx.z * HPW;
  const int nh = min(HPW, rep - h0);
  const int q0 = qb * 64 + wave * 16;
  if (q0 >= T) return;
  const int* pt = kv.page_table + (size_t)(sblk * rm.seq_stride) * kv.pages_per_seq;
  const size_t row0 = (size_t)sblk * T;
  const int qpos = min(q0 + qcol, T - 1);   // columns past T repeat the last position and are not stored
  const size_t qstride = (size_t)n_q_heads * HD;
  Frag qf[HPW][KK];
#pragma unroll
  for (int h = 0; h < HPW; ++h)
    if (h < nh) {
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        qf[h][kk].u = *(const uint4*)(q + (row0 + qpos) * qstride + (size_t)(kvh * rep + h0 + h) * HD + kk * 32 + grp * 8);
    }
  float m_run[HPW], l_run[HPW];
  f32x4 o[HPW][DT];
#pragma unroll
  for (int h = 0; h < HPW; ++h) {
    m_run[h] = -INFINITY; l_run[h] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[h][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float scale2 = 1.4426950408889634f / sqrtf((float)HD);   // scores in units of log2
  const int q_hi = min(q0 + 15, T - 1);
  const int npairs = q_hi / 32 + 1;
  const int last_page = q_hi / kPageTokens;
  const bf16* kpool = (const bf16*)kv.k;
  const bf16* vpool = (const bf16*)kv.v;
  const size_t page_elems = (size_t)hkv * kPageTokens * HD;
  for (int pp = 0; pp < npairs; ++pp) {
    const int pa = pt[2 * pp];
    const int pb = pt[min(2 * pp + 1, last_page)];
    Frag kf[2][KK], vf[DT];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = lane & 15;
      const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);   // key row r of score tile t
      const bf16* kp = kpool + (size_t)(ptok < 16 ? pa : pb) * page_elems + ((size_t)kvh * kPageTokens + (ptok & 15)) * HD;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[t][kk].u = *(const uint4*)(kp + kk * 32 + grp * 8);
    }
    const bf16* vp = vpool + (size_t)(grp < 2 ? pa : pb) * page_elems + (size_t)kvh * HD * kPageTokens + (grp & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[dt].u = *(const uint4*)(vp + (size_t)(dt * 16 + (lane & 15)) * kPageTokens);
    const bool diag = pp * 32 + 31 > q0;   // some (query, key) of the pair is masked
#pragma unroll
    for (int h = 0; h < HPW; ++h) {
      if (h >= nh) continue;
      f32x4 sc[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) sc[t] = mfma16(kf[t][kk], qf[h][kk], sc[t]);
      }
      // lane (query qcol, group grp) holds keys pp*32 + 8 grp + e, e = 4 t + j
      float p[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = sc[e >> 2][e & 3] * scale2;
      if (diag) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (pp * 32 + 8 * grp + e > qpos) p[e] = -INFINITY;
      }
      float m_loc = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
      m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 16, 64));
      m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, 64));
      const float m_new = fmaxf(m_run[h], m_loc);   // finite: key 0 is visible to every query
      const float alpha = exp2f(m_run[h] - m_new);
      float psum = 0.f;
      Frag pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = exp2f(p[e] - m_new);
        psum += pe;
        pf.v[e] = (bf16)pe;
      }
      l_run[h] = l_run[h] * alpha + psum;
      m_run[h] = m_new;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
        for (int j = 0; j < 4; ++j) o[h][dt][j] *= alpha;
        o[h][dt] = mfma16(vf[dt], pf, o[h][dt]);
      }
    }
  }
  if (q0 + qcol >= T) return;
#pragma unroll
  for (int h = 0; h < HPW; ++h) {
    if (h >= nh) continue;
    float l = l_run[h];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
    bf16* op = out + (row0 + qpos) * qstride + (size_t)(kvh * rep + h0 + h) * HD + grp * 4;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      bf16x4 ov;
#pragma unroll
      for (int j = 0; j < 4; ++j) ov[j] = (bf16)(o[h][dt][j] * inv);
      *(bf16x4*)(op + dt * 16) = ov;
    }
  }
}

hipError_t m_flash_attention(const void* q, RowMap rm, KVCache kv, void* out, int n_seq, int n_q_heads, hipStream_t st) {
  if (n_seq == 0) return hipSuccess;
  const int rep = n_q_heads / kv.n_kv_heads;
  const int nqb = (rm.T + 63) / 64;
  if (kv.head_dim == 64) {
    constexpr int HPW = 7;
    dim3 grid(nqb, n_seq * kv.n_kv_heads, (rep + HPW - 1) / HPW);
    return launch(KID_FLASH_ATTN, k_flash_attention<64, HPW>, grid, dim3(256), 0, st, (const bf16*)q, rm, kv, (bf16*)out, n_q_heads);
  }
  if (kv.head_dim == 128) {
    constexpr int HPW = 3;
    dim3 grid(nqb, n_seq * kv.n_kv_heads, (rep + HPW - 1) / HPW);
    return launch(KID_FLASH_ATTN, k_flash_attention<128, HPW>, grid, dim3(256), 0, st, (const bf16*)q, rm, kv, (bf16*)out, n_q_heads);
  }
  return hipErrorInvalidValue;
}

}  // namespace sapo
