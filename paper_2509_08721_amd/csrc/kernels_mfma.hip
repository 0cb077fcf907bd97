// bf16 MFMA kernels for gfx950: weight packing, the token-parallel ("big") GEMM used by prefill and
// scoring, the 64-token weight-streaming ("skinny") GEMM used by decode, the fused LM-head kernels
// (log-softmax + Gumbel-max sampler, log-softmax + target gather) and paged GQA decode attention.
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
  ProfScope prof_(KID_MISC, st);
  const size_t total = (size_t)(n_rows / 32) * (K / 16) * 64;
  if (total == 0) return hipSuccess;
  k_pack_weight<<<(unsigned)((total + 255) / 256), 256, 0, st>>>((const bf16*)src, n_rows, K, (uint4*)dst, dst_tile0,
                                                                  dst_tile_stride);
  return hipGetLastError();
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
  ProfScope prof_(KID_GEMM_BIG, st);
  if (M == 0) return hipSuccess;
  dim3 grid(N / 128, (M + 255) / 256);
  k_gemm_big<<<grid, 256, 0, st>>>((const bf16*)X, ldx, (const uint4*)Wp, M, N, K, epi);
  return hipGetLastError();
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
  hipError_t e;
  {
    ProfScope prof_(KID_LMHEAD_SCORE, st);
    k_lmhead_score<<<grid, 256, 0, st>>>((const bf16*)X, (const uint4*)Wp, max_rows, n_rows_dev, V, K, row_seq_pos,
                                         tokens, T, partials);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  ProfScope prof2_(KID_LMHEAD_SCORE_MERGE, st);
  k_lmhead_score_merge<<<(max_rows + 255) / 256, 256, 0, st>>>(partials, max_rows, n_rows_dev, row_seq_pos, T,
                                                               out_logprobs);
  return hipGetLastError();
}

// =======================================================================================
// Skinny GEMM (decode): up to 64 tokens, weights streamed once from HBM.
// 512 threads = 8 waves.  A workgroup owns one 32-feature tile (a gate/up tile pair for SwiGLU)
// over a k range of at most kChunkSteps steps; the 8 waves split the k steps (wave w takes steps
// w, w+8, ...) and their partial 32x64 tiles are summed through LDS in a fixed order (waves 4..7
// into 0..3, then 0..3 by all threads).  When K is split over several workgroups, each writes its
// partial tile to scratch and the last one to arrive (atomic counter per tile) sums all partials in
// k order, so results never depend on scheduling.  Weight fragments are requested before X is
// staged: they do not depend on it.
// X (64 tokens x k range) sits in LDS in fragment order; it comes from an X-packed bf16 buffer, or
// from the fp32 residual stream, RMS-normalised on the way in with the row sums of squares that the
// producing kernel left behind (ssq[part][token], summed here).
// After the reduction thread t owns, for token (t/256)*32 + lane%32 (lane = t % 64), the four
// features (lane/32)*4 + 8 i + (0..3) of the tile, i = (t / 64) % 4.
// ---------------------------------------------------------------------------------------
constexpr int kChunkSteps = 56;                                  // 896 k per workgroup
constexpr int kSkinnyXBytes = kChunkSteps * 2 * 64 * 16;         // 114688
constexpr int kSkinnyPartBytes = 4 * 32 * 64 * 4;                // 32768
constexpr int kSkinnyLds = kSkinnyXBytes + kSkinnyPartBytes;

__device__ __forceinline__ void skinny_load_w(const uint4* __restrict__ Wp, int KS, int tile, int ks_begin, int ks_end,
                                              Frag (&w)[7]) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint4* wb = Wp + (size_t)tile * KS * 64 + lane;
#pragma unroll
  for (int i = 0; i < 7; ++i) {
    const int ks = ks_begin + wave + 8 * i;
    if (ks < ks_end) w[i].n = __builtin_nontemporal_load((const u32x4*)(wb + (size_t)ks * 64));
  }
}

// Stage k steps [ks_begin, ks_end) of X into LDS (fragment order, local step index).
// `part` is used as scratch for the per-token scales in h mode.
__device__ __forceinline__ void skinny_stage_x(const SkinnyIn& in, int n_rows, int K, int ks_begin, int ks_end,
                                               uint4* xs, float* part) {
  const int tid = threadIdx.x;
  const int nks = ks_end - ks_begin;
  if (in.xp) {
    // contiguous copy, 8 loads in flight per thread
    const uint4* src = (const uint4*)in.xp + (size_t)ks_begin * 128;
    const int total = nks * 128;
    for (int base = 0; base < total; base += 512 * 8) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * 512 + tid;
        if (i < total) v[u] = src[i];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * 512 + tid;
        if (i < total) xs[i] = v[u];
      }
    }
  } else {
    float* scale = part;
    if (tid < 64) {
      float s = 0.f;
      if (tid < n_rows)
        for (int p = 0; p < in.ssq_parts; ++p) s += in.ssq[(size_t)p * 64 + tid];
      scale[tid] = (tid < n_rows) ? 1.0f / sqrtf(s / (float)K + in.eps) : 0.f;
    }
    __syncthreads();
    const int k0 = ks_begin * 16, nk4 = nks * 4;      // float4 groups per row in this range
    const float inv_nk4 = 1.0f / (float)nk4;
    const int total = 64 * nk4;
    bf16* xb = (bf16*)xs;
    for (int base = 0; base < total; base += 512 * 8) {
      float4 v[8], g[8];
      int tk[8], kk[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * 512 + tid;
        tk[u] = (int)(((float)i + 0.5f) * inv_nk4);
        kk[u] = (i - tk[u] * nk4) * 4;
        if (i < total && tk[u] < n_rows) {
          v[u] = *(const float4*)(in.h + (size_t)tk[u] * K + k0 + kk[u]);
          g[u] = *(const float4*)(in.gain + k0 + kk[u]);
        } else {
          v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
          g[u] = v[u];
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * 512 + tid;
        if (i < total) {
          const float sc = scale[tk[u]];
          bf16x4 o;
          o[0] = (bf16)(v[u].x * sc * g[u].x); o[1] = (bf16)(v[u].y * sc * g[u].y);
          o[2] = (bf16)(v[u].z * sc * g[u].z); o[3] = (bf16)(v[u].w * sc * g[u].w);
          *(bf16x4*)(xb + xpack_index(tk[u], kk[u])) = o;
        }
      }
    }
    __syncthreads();   // scale[] lives in `part`, which the reduction reuses
  }
}

__device__ __forceinline__ void skinny_mma(const Frag (&w)[7], int nks, const uint4* xs, f32x16& acc0, f32x16& acc1) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 7; ++i) {
    const int ks = wave + 8 * i;     // local step
    if (ks < nks) {
      Frag x0, x1;
      x0.u = xs[(ks * 2 + 0) * 64 + lane];
      x1.u = xs[(ks * 2 + 1) * 64 + lane];
      acc0 = mfma32(w[i], x0, acc0);
      acc1 = mfma32(w[i], x1, acc1);
    }
  }
}

// Cross-wave reduction of the 8 partial tiles; thread t gets its four values in out[4].
__device__ __forceinline__ void skinny_reduce(f32x16& acc0, f32x16& acc1, float* part, float (&out)[4]) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  __syncthreads();
  if (wave >= 4) {
    float* p = part + (size_t)(wave - 4) * 2048 + lane;
#pragma unroll
    for (int v = 0; v < 16; ++v) { p[v * 64] = acc0[v]; p[(16 + v) * 64] = acc1[v]; }
  }
  __syncthreads();
  if (wave < 4) {
    float* p = part + (size_t)wave * 2048 + lane;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] += p[v * 64]; acc1[v] += p[(16 + v) * 64]; }
  }
  __syncthreads();
  if (wave < 4) {
    float* p = part + (size_t)wave * 2048 + lane;
#pragma unroll
    for (int v = 0; v < 16; ++v) { p[v * 64] = acc0[v]; p[(16 + v) * 64] = acc1[v]; }
  }
  __syncthreads();
  const int vq = tid >> 6;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float* p = part + (size_t)(vq * 4 + j) * 64 + lane;
    out[j] = (p[0] + p[2048]) + (p[2 * 2048] + p[3 * 2048]);
  }
}

__global__ void __launch_bounds__(512) k_gemm_skinny(SkinnyIn in, const uint4* __restrict__ Wp, int n_rows, int N, int K,
                                                     SkinnyEpi ep, int ksplit) {
  extern __shared__ uint4 dyn_smem[];
  __shared__ int s_last;
  uint4* xs = dyn_smem;
  float* part = (float*)((char*)dyn_smem + kSkinnyXBytes);
  const int tid = threadIdx.x, lane = tid & 63, vq = tid >> 6;
  const int KS = K >> 4;
  const int unit = blockIdx.x / ksplit, c = blockIdx.x % ksplit;
  const int per = (KS + ksplit - 1) / ksplit;
  const int ks_begin = c * per, ks_end = min(KS, ks_begin + per);
  const int nks = ks_end - ks_begin;
  const int nt = (ep.mode == SK_SWIGLU) ? 2 : 1;
  const int tile0 = unit * nt;

  Frag w0[7], w1[7];
  skinny_load_w(Wp, KS, tile0, ks_begin, ks_end, w0);
  if (nt == 2) skinny_load_w(Wp, KS, tile0 + 1, ks_begin, ks_end, w1);
  skinny_stage_x(in, n_rows, K, ks_begin, ks_end, xs, part);
  __syncthreads();

  const int tok = (vq >> 2) * 32 + (lane & 31);
  const int fsub = (lane >> 5) * 4 + 8 * (vq & 3);
  float r[4], gate[4];
  for (int t = 0; t < nt; ++t) {
    f32x16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
    skinny_mma(t == 0 ? w0 : w1, nks, xs, acc0, acc1);
    skinny_reduce(acc0, acc1, part, r);
    if (t == 0 && nt == 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) gate[j] = r[j];
    }
  }
  const int tile = tile0;
  if (ksplit > 1) {
    // split-K fix-up: publish the partial, the last workgroup of the tile sums all of them in k order
    float* my = ep.scratch + ((size_t)tile * ksplit + c) * 2048 + tid * 4;
    *(float4*)my = make_float4(r[0], r[1], r[2], r[3]);
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      const int old = atomicAdd(ep.counters + tile, 1);
      s_last = (old == ksplit - 1) ? 1 : 0;
      if (s_last) ep.counters[tile] = 0;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    // the fence above made the other workgroups' partials visible (L1 invalidated): plain loads
    float4 pv[8];
#pragma unroll
    for (int cc = 0; cc < 8; ++cc)
      pv[cc] = (cc < ksplit) ? *(const float4*)(ep.scratch + ((size_t)tile * ksplit + cc) * 2048 + tid * 4)
                             : make_float4(0.f, 0.f, 0.f, 0.f);
    r[0] = r[1] = r[2] = r[3] = 0.f;
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) { r[0] += pv[cc].x; r[1] += pv[cc].y; r[2] += pv[cc].z; r[3] += pv[cc].w; }
  }
  if (ep.mode == SK_SWIGLU) {
    const int fidx = (tile >> 1) * 32 + fsub;
    bf16x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (tok < n_rows) ? (bf16)(silu_f(gate[j]) * r[j]) : (bf16)0.f;
    *(bf16x4*)(ep.out_xp + xpack_index(tok, fidx)) = o;
    return;
  }
  float ss = 0.f;
  if (tok < n_rows) {
    float4* p = (float4*)(ep.out_f32 + (size_t)tok * ep.ldc + tile * 32 + fsub);
    float4 v = make_float4(r[0], r[1], r[2], r[3]);
    if (ep.mode == SK_ADD_F32) {
      const float4 o = *p;
      v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
    }
    *p = v;
    ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  if (ep.ssq_out) {
    // sum of squares of the tile's 32 features per token: 8 threads per token, fixed order
    __syncthreads();
    part[tid] = ss;
    __syncthreads();
    if (tid < 64) {
      const int ti = tid >> 5, l31 = tid & 31;
      float s = 0.f;
      for (int q = 0; q < 4; ++q)
        for (int hf = 0; hf < 2; ++hf) s += part[(ti * 4 + q) * 64 + hf * 32 + l31];
      ep.ssq_out[(size_t)tile * 64 + tid] = s;
    }
  }
}

hipError_t m_gemm_skinny(SkinnyIn in, const void* Wp, int n_rows, int N, int K, SkinnyEpi epi, int ksplit,
                         hipStream_t st) {
  ProfScope prof_(KID_GEMM_SKINNY, st);
  const int KS = K / 16;
  if (ksplit < 1 || (KS + ksplit - 1) / ksplit > kChunkSteps || (ksplit - 1) * ((KS + ksplit - 1) / ksplit) >= KS ||
      (ksplit > 1 && (epi.mode == SK_SWIGLU || !epi.scratch || !epi.counters)))
    return hipErrorInvalidValue;
  const int n_tiles = N / 32;
  const int units = (epi.mode == SK_SWIGLU) ? n_tiles / 2 : n_tiles;
  k_gemm_skinny<<<units * ksplit, 512, kSkinnyLds, st>>>(in, (const uint4*)Wp, n_rows, N, K, epi, ksplit);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// LM head for decode: logits tile -> online log-sum-exp + Gumbel-max, logits never stored.
// Same skinny tile engine over the full K; each workgroup walks a contiguous range of vocabulary
// tiles (next tile's weights in flight while the current one is reduced) keeping, per thread, the
// running (max, sum exp) and best perturbed score of its token; per-workgroup results go to
// `partials` [n_wg][64][5] and a second kernel merges them in a fixed order.
// Row r of X is sequence seq0 + r.
// ---------------------------------------------------------------------------------------
constexpr int kSampleWgs = 256;
size_t m_lmhead_sample_partial_floats() { return (size_t)kSampleWgs * 64 * 5; }

__global__ void __launch_bounds__(512) k_lmhead_sample(SkinnyIn in, const uint4* __restrict__ Wp, int n_rows, int seq0,
                                                       int V, int K, SampleParams sp, float* __restrict__ partials) {
  extern __shared__ uint4 dyn_smem[];
  uint4* xs = dyn_smem;
  float* part = (float*)((char*)dyn_smem + kSkinnyXBytes);
  const int tid = threadIdx.x, lane = tid & 63, vq = tid >> 6;
  const int KS = K >> 4;
  const int n_tiles = V >> 5;
  const int per = (n_tiles + gridDim.x - 1) / gridDim.x;
  const int t_begin = blockIdx.x * per, t_end = min(n_tiles, t_begin + per);
  Frag wa[7], wb[7];
  if (t_begin < t_end) skinny_load_w(Wp, KS, t_begin, 0, KS, wa);
  skinny_stage_x(in, n_rows, K, 0, KS, xs, part);
  __syncthreads();
  const int tok = (vq >> 2) * 32 + (lane & 31);
  const int fsub = (lane >> 5) * 4 + 8 * (vq & 3);
  resolve_sample_params(sp);
  const int step = *sp.step;
  const bool noisy = sp.temperature != 0.f;
  LseAcc lse; lse.init();
  BestAcc best; best.init();
  for (int tile = t_begin; tile < t_end; ++tile) {
    if (tile + 1 < t_end) skinny_load_w(Wp, KS, tile + 1, 0, KS, wb);
    f32x16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
    skinny_mma(wa, KS, xs, acc0, acc1);
    float r[4];
    skinny_reduce(acc0, acc1, part, r);
    const int v0 = tile * 32 + fsub;
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (noisy) gumbel4(sp.seed_lo, sp.seed_hi, (uint32_t)(seq0 + tok), (uint32_t)step, (uint32_t)(v0 >> 2), g);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lse.add(r[j]);
      const float y = noisy ? r[j] / sp.temperature + g[j] : r[j];
      best.add(y, r[j], v0 + j);
    }
#pragma unroll
    for (int i = 0; i < 7; ++i) wa[i] = wb[i];
  }
  // combine the 8 threads that share a token (fixed order), one thread per token writes
  __syncthreads();
  float* sm = part;   // [5][512]
  sm[tid] = lse.m; sm[512 + tid] = lse.l; sm[1024 + tid] = best.y; sm[1536 + tid] = best.z;
  ((int*)sm)[2048 + tid] = best.id;
  __syncthreads();
  if (tid < 64) {
    const int ti = tid >> 5, l31 = tid & 31;
    LseAcc a; a.init();
    BestAcc b; b.init();
    for (int q = 0; q < 4; ++q)
      for (int hf = 0; hf < 2; ++hf) {
        const int t = (ti * 4 + q) * 64 + hf * 32 + l31;
        a.merge(sm[t], sm[512 + t]);
        b.add(sm[1024 + t], sm[1536 + t], ((int*)sm)[2048 + t]);
      }
    float* p = partials + ((size_t)blockIdx.x * 64 + tid) * 5;
    p[0] = a.m; p[1] = a.l; p[2] = b.y; p[3] = b.z; ((int*)p)[4] = b.id;
  }
}

__global__ void k_lmhead_sample_merge(const float* __restrict__ partials, int n_wg, int n_rows, int seq0, SampleParams sp) {
  const int r = blockIdx.x;
  const int lane = threadIdx.x;
  if (r >= n_rows) return;
  LseAcc a; a.init();
  BestAcc b; b.init();
  for (int w = lane; w < n_wg; w += 64) {
    const float* p = partials + ((size_t)w * 64 + r) * 5;
    a.merge(p[0], p[1]);
    b.add(p[2], p[3], ((const int*)p)[4]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    a.merge(__shfl_xor(a.m, o, 64), __shfl_xor(a.l, o, 64));
    b.add(__shfl_xor(b.y, o, 64), __shfl_xor(b.z, o, 64), __shfl_xor(b.id, o, 64));
  }
  if (lane == 0) {
    const int step = *sp.step;
    const size_t o = (size_t)(seq0 + r) * sp.max_new + step;
    sp.out_tokens[o] = b.id;
    sp.out_logprobs[o] = b.z - (a.m + logf(a.l));
  }
}

hipError_t m_lmhead_sample(SkinnyIn in, const void* Wp, int n_rows, int seq0, int V, int K, SampleParams sp,
                           float* partials, hipStream_t st) {
  if (K / 16 > kChunkSteps) return hipErrorInvalidValue;
  int n_wg = kSampleWgs;
  const int n_tiles = V / 32;
  if (n_wg > n_tiles) n_wg = n_tiles;
  hipError_t e;
  {
    ProfScope prof_(KID_LMHEAD_SAMPLE, st);
    k_lmhead_sample<<<n_wg, 512, kSkinnyLds, st>>>(in, (const uint4*)Wp, n_rows, seq0, V, K, sp, partials);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  ProfScope prof2_(KID_LMHEAD_SAMPLE_MERGE, st);
  k_lmhead_sample_merge<<<n_rows, 64, 0, st>>>(partials, n_wg, n_rows, seq0, sp);
  return hipGetLastError();
}

// Kernels that use more than 64 KiB of LDS need the limit raised once per process.
hipError_t m_init_attributes() {
  hipError_t e = hipFuncSetAttribute((const void*)k_gemm_skinny, hipFuncAttributeMaxDynamicSharedMemorySize, kSkinnyLds);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void*)k_lmhead_sample, hipFuncAttributeMaxDynamicSharedMemorySize, kSkinnyLds);
}

// Decode-side embedding gather: h[m, :] = embed[token(m), :] plus the row's sum of squares
// (ssq[m], one part) for the norm that the first GEMM folds in.
__global__ void __launch_bounds__(256) k_embed_ssq(const int32_t* __restrict__ tokens, int tok_stride, const int* step,
                                                   const bf16* __restrict__ embed, float* __restrict__ h,
                                                   float* __restrict__ ssq, int d) {
  const int m = blockIdx.x;
  const int tok = tokens[(size_t)m * tok_stride + (*step - 1)];
  const bf16* e = embed + (size_t)tok * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float v = (float)e[i];
    h[(size_t)m * d + i] = v;
    ss += v * v;
  }
  __shared__ float red[4];
  ss = wave_reduce_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssq[m] = (red[0] + red[1]) + (red[2] + red[3]);
}
hipError_t m_embed_ssq(const int32_t* tokens, int tok_stride, const int* step, const void* embed, float* h, float* ssq,
                       int M, int d, hipStream_t st) {
  ProfScope prof_(KID_EMBED, st);
  k_embed_ssq<<<M, 256, 0, st>>>(tokens, tok_stride, step, (const bf16*)embed, h, ssq, d);
  return hipGetLastError();
}

// Sum of squares of each row of h [M, d] -> ssq[m].
__global__ void __launch_bounds__(256) k_row_ssq(const float* __restrict__ h, float* __restrict__ ssq, int d) {
  const int m = blockIdx.x;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float v = h[(size_t)m * d + i]; ss += v * v; }
  __shared__ float red[4];
  ss = wave_reduce_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssq[m] = (red[0] + red[1]) + (red[2] + red[3]);
}
hipError_t m_row_ssq(const float* h, float* ssq, int M, int d, hipStream_t st) {
  ProfScope prof_(KID_MISC, st);
  k_row_ssq<<<M, 256, 0, st>>>(h, ssq, d);
  return hipGetLastError();
}

// =======================================================================================
// Decode attention over the paged KV cache, fused with rotary + KV append of the new token.
// One workgroup (4 waves) per (sequence, KV head); all query heads of the group ride together as
// the 16 columns of 16x16x32 MFMAs.  S^T = K Q^T (tokens x queries) so that each lane owns one
// query column: the running max / sum are per-lane scalars plus two cross-lane shuffles, and the
// probabilities a lane produces are exactly its operand of O^T = V^T P^T.  Token rows are permuted
// inside a 32-token page pair so that a lane's 8 probabilities are 8 consecutive tokens, which is
// what the token-minor V page delivers in one 16-byte load.  Waves take page pairs round-robin and
// are merged through LDS.
// ---------------------------------------------------------------------------------------
template <int HD>
__global__ void __launch_bounds__(256) k_decode_attention(const float* __restrict__ qkv, const float2* __restrict__ rope,
                                                          RowMap rm, KVCache kv, bf16* __restrict__ out, int out_xp,
                                                          int n_q_heads) {
  constexpr int KK = HD / 32;   // k steps of S^T = K Q^T
  constexpr int DT = HD / 16;   // 16-row tiles of O^T
  __shared__ __attribute__((aligned(16))) bf16 qs[16 * HD];
  __shared__ float sm_m[4][16], sm_l[4][16];
  __shared__ float sm_o[4][HD][16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hkv = kv.n_kv_heads, rep = n_q_heads / hkv;
  const int s = blockIdx.x / hkv, kvh = blockIdx.x % hkv;
  int seq, pos;
  rm.get(s, seq, pos);
  const int ctx = pos + 1;
  const int* pt = kv.page_table + (size_t)seq * kv.pages_per_seq;
  bf16* kpool = (bf16*)kv.k;
  bf16* vpool = (bf16*)kv.v;
  const size_t page_elems = (size_t)hkv * kPageTokens * HD;
  // ---- rotary on the group's queries and the new key; append key / value -------------------
  {
    const int half = HD / 2;
    const float* row = qkv + (size_t)s * (n_q_heads + 2 * hkv) * HD;
    const int page = pt[pos / kPageTokens], slot = pos % kPageTokens;
    for (int idx = tid; idx < 16 * half; idx += 256) {
      const int r = idx / half, i = idx % half;
      float r1 = 0.f, r2 = 0.f;
      if (r < rep) {
        const float* x = row + (size_t)(kvh * rep + r) * HD;
        const float2 cs = rope[(size_t)pos * half + i];
        r1 = x[i] * cs.x - x[i + half] * cs.y;
        r2 = x[i + half] * cs.x + x[i] * cs.y;
      }
      qs[r * HD + i] = (bf16)r1;
      qs[r * HD + i + half] = (bf16)r2;
    }
    for (int i = tid; i < half; i += 256) {
      const float* x = row + (size_t)(n_q_heads + kvh) * HD;
      const float2 cs = rope[(size_t)pos * half + i];
      bf16* kp = kpool + (size_t)page * page_elems + ((size_t)kvh * kPageTokens + slot) * HD;
      kp[i] = (bf16)(x[i] * cs.x - x[i + half] * cs.y);
      kp[i + half] = (bf16)(x[i + half] * cs.x + x[i] * cs.y);
    }
    for (int i = tid; i < HD; i += 256) {
      const float* x = row + (size_t)(n_q_heads + hkv + kvh) * HD;
      vpool[(size_t)page * page_elems + ((size_t)kvh * HD + i) * kPageTokens + slot] = (bf16)x[i];
    }
  }
  __threadfence();
  __syncthreads();
  const int qcol = lane & 15, grp = lane >> 4;
  Frag qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk].u = *(const uint4*)(qs + qcol * HD + kk * 32 + grp * 8);
  const float scale = 1.0f / sqrtf((float)HD);
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int npairs = (ctx + 31) / 32;
  const int last_page = (ctx - 1) / kPageTokens;
  for (int pp = wave; pp < npairs; pp += 4) {
    const int pa = pt[2 * pp];
    const int pb = pt[min(2 * pp + 1, last_page)];
    // key rows of the two score tiles: tile t row r is pair-token 8 (r / 4) + 4 t + r % 4
    f32x4 sc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = lane & 15;
      const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);
      const bf16* kp = kpool + (size_t)(ptok < 16 ? pa : pb) * page_elems + ((size_t)kvh * kPageTokens + (ptok & 15)) * HD;
      sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        Frag kf;
        kf.u = *(const uint4*)(kp + kk * 32 + grp * 8);
        sc[t] = mfma16(kf, qf[kk], sc[t]);
      }
    }
    // lane (query qcol, group grp) now holds pair-tokens 8 grp + e, e = 4 t + j
    float p[8];
    float m_loc = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int n = pp * 32 + 8 * grp + e;
      const float sv = sc[e >> 2][e & 3] * scale;
      p[e] = (n < ctx) ? sv : -INFINITY;
      m_loc = fmaxf(m_loc, p[e]);
    }
    m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 16, 64));
    m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, 64));
    const float m_new = fmaxf(m_run, m_loc);
    const float alpha = __expf(m_run - m_new);
    float psum = 0.f;
    Frag pf;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float pe = __expf(p[e] - m_new);
      psum += pe;
      pf.v[e] = (bf16)pe;
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    // O^T += V^T P^T ; V page is [hd][16 tokens]: tokens 8 grp .. 8 grp + 7 of the pair
    const bf16* vp = vpool + (size_t)(grp < 2 ? pa : pb) * page_elems + (size_t)kvh * HD * kPageTokens + (grp & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      Frag vf;
      vf.u = *(const uint4*)(vp + (size_t)(dt * 16 + (lane & 15)) * kPageTokens);
#pragma unroll
      for (int j = 0; j < 4; ++j) o[dt][j] *= alpha;
      o[dt] = mfma16(vf, pf, o[dt]);
    }
  }
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (grp == 0) { sm_m[wave][qcol] = m_run; sm_l[wave][qcol] = l_run; }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) sm_o[wave][dt * 16 + grp * 4 + j][qcol] = o[dt][j];
  __syncthreads();
  for (int idx = tid; idx < 16 * HD; idx += 256) {
    const int q = idx & 15, d = idx >> 4;
    if (q >= rep) continue;
    float mx = fmaxf(fmaxf(sm_m[0][q], sm_m[1][q]), fmaxf(sm_m[2][q], sm_m[3][q]));
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = __expf(sm_m[w][q] - mx);
      num += wgt * sm_o[w][d][q];
      den += wgt * sm_l[w][q];
    }
    const int col = (kvh * rep + q) * HD + d;
    const bf16 val = (bf16)(num / den);
    if (out_xp) out[xpack_index(s, col)] = val;
    else out[(size_t)s * n_q_heads * HD + col] = val;
  }
}

hipError_t m_decode_attention(const float* qkv, const float2* rope, RowMap rm, KVCache kv, bf16* out, int out_xp, int S,
                              int n_q_heads, hipStream_t st) {
  ProfScope prof_(KID_DECODE_ATTN, st);
  const int grid = S * kv.n_kv_heads;
  if (kv.head_dim == 64)
    k_decode_attention<64><<<grid, 256, 0, st>>>(qkv, rope, rm, kv, out, out_xp, n_q_heads);
  else if (kv.head_dim == 128)
    k_decode_attention<128><<<grid, 256, 0, st>>>(qkv, rope, rm, kv, out, out_xp, n_q_heads);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace sapo
