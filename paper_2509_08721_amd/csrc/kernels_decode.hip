// Decode-side 16-bit MFMA kernels for gfx950 (one new token per sequence and step).  Operands are
// IEEE half: packed weights hold the model's bf16 values converted to half, activations are rounded
// to half (see the note at the top of kernels_mfma.hip).
//
// Every projection of a decode step is a "skinny" GEMM: few tokens (64 per block), all weights
// streamed once from HBM.  The kernels here are built around v_mfma_f32_16x16x32_f16 with both
// operands already in fragment order in global memory, so that a wave's operand load is one
// contiguous 1 KiB read that goes straight into registers:
//   weights  W16[((tile * KS + ks) * 64 + lane)]           (uint4 = 8 half)
//            = W[tile*16 + lane%16][ks*32 + (lane/16)*8 .. +7],                       KS = K / 32
//   tokens   X16[(((tok/64) * KS + ks) * 4 + (tok/16)%4) * 64 + tok%16 + 16*((k%32)/8)]
//            = x[tok][ks*32 + ((k%32)/8)*8 .. +7]
// D = W-fragment x X-fragment leaves lane l with features (l/16)*4 .. +3 of token l%16.
//
// RMSNorm never runs on its own: the kernel that produces the residual stream also writes
// half(h * gain) in X16 order plus per-tile sums of squares of h, and the GEMM that consumes it
// multiplies its accumulators by rsqrt(mean(h^2) + eps) (the scale is per token, so it commutes
// with the contraction).
#include "common.h"
#include "coherent.h"

namespace sapo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
union Frag16 {
  uint4 u;
  u32x4 n;
  bf16x8 v;
  f16x8 h;
};

__device__ __forceinline__ f32x4 mfma16(const Frag16& a, const Frag16& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c, 0, 0, 0);
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// uint4 index of the chunk that holds x[tok][k .. k+7] (k a multiple of 8) in X16 order.
__host__ __device__ __forceinline__ size_t x16_chunk(int tok, int k, int KS) {
  return ((((size_t)(tok >> 6) * KS + (k >> 5)) * 4 + ((tok >> 4) & 3)) * 64) + (tok & 15) + 16 * ((k >> 3) & 3);
}

// ---------------------------------------------------------------------------------------
// weight packing: row-major bf16 [n_rows, K] -> half, W16 order; 16-row tile t goes to tile slot
// tile0 + t * tile_stride (stride 2 interleaves gate and up tiles).
// ---------------------------------------------------------------------------------------
__global__ void k_pack_weight16(const bf16* __restrict__ src, int n_rows, int K, uint4* __restrict__ dst, int tile0,
                                int tile_stride) {
  const int KS = K >> 5;
  const size_t total = (size_t)(n_rows >> 4) * KS * 64;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const int ks = (int)((idx >> 6) % KS);
  const int t = (int)((idx >> 6) / KS);
  const int row = t * 16 + (lane & 15), k = ks * 32 + (lane >> 4) * 8;
  Frag16 v, o;
  v.u = *(const uint4*)(src + (size_t)row * K + k);
#pragma unroll
  for (int e = 0; e < 8; ++e) o.h[e] = from_f32<f16>((float)v.v[e]);   // bf16 value -> half
  dst[((size_t)(tile0 + t * tile_stride) * KS + ks) * 64 + lane] = o.u;
}
hipError_t d_pack_weight16(const void* src, int n_rows, int K, void* dst, int dst_tile0, int dst_tile_stride,
                           hipStream_t st) {
  const size_t total = (size_t)(n_rows / 16) * (K / 32) * 64;
  if (total == 0) return hipSuccess;
  return launch(KID_MISC, k_pack_weight16, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16*)src, n_rows, K, (uint4*)dst, dst_tile0,
                                                                    dst_tile_stride);
}

// ---------------------------------------------------------------------------------------
// Sum of the ssq parts of one token, spread over the 8 waves of a workgroup: thread (grp, tok)
// loads parts grp, grp + 8, ... early (ssq_issue) and the sums meet in LDS later (ssq_finish).
// ---------------------------------------------------------------------------------------
constexpr int kSsqPerThread = 12;   // up to 96 parts

// ssq is not null and parts >= 1.  Every thread asks for all kSsqPerThread values, a part past the end being the last
// part again (dropped in ssq_publish): with a request under a branch each, the compiler waited for the first one on
// the spot - a memory round trip in front of the kernel's weight requests.
__device__ __forceinline__ void ssq_issue(const float* __restrict__ ssq, int parts, int stride, int tok0,
                                          float (&sq)[kSsqPerThread]) {
  const int tok = threadIdx.x & 63, grp = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < kSsqPerThread; ++i) sq[i] = ssq[(size_t)min(grp + 8 * i, parts - 1) * stride + tok0 + tok];
}
// s_part: LDS [8][64].  Call before a __syncthreads(); ssq_scale() after it.
__device__ __forceinline__ void ssq_publish(const float (&sq)[kSsqPerThread], int parts, float* s_part) {
  const int grp = threadIdx.x >> 6;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kSsqPerThread; ++i) s += (grp + 8 * i < parts) ? sq[i] : 0.f;
  s_part[threadIdx.x] = s;
}
__device__ __forceinline__ float ssq_scale(const float* s_part, int tok_local, int norm_dim, float eps) {
  float s = 0.f;
#pragma unroll
  for (int g = 0; g < 8; ++g) s += s_part[g * 64 + tok_local];
  return 1.0f / sqrtf(s / (float)norm_dim + eps);
}

// ---------------------------------------------------------------------------------------
// Skinny GEMM.  512 threads = 8 waves per workgroup.
// A workgroup owns NT 16-feature tiles x TG 16-token groups over the whole K; wave w takes the
// k steps w, w + 8, ... (R of them per round, all loads of a round in flight at once), and the
// 8 partial results are summed through LDS in wave order, so results never depend on timing.
// Small per-workgroup operands matter more than the number of workgroups: a compute unit ingests
// roughly 100 GB/s, so a 64-token block is split into 4 / TG workgroups per tile, which re-read
// the tile's weights from the L2 they share (block ids are laid out so that they land on the
// same XCD: ids that differ by a multiple of 8).
// Epilogues:
//   STORE  : out_f32[tok][feat] = acc * scale(tok)
//   SWIGLU : tiles come in (gate, up) pairs; act = silu(gate * scale) * (up * scale) -> half, X16 order
//   RESID  : h[tok][feat] += acc;  xp_out = half(h * gain_next) in X16 order;  ssq_out[tile][tok] =
//            sum of h^2 over the tile's 16 features
// ---------------------------------------------------------------------------------------
template <int NT, int TG, int R, int MODE>
// The first arguments are passed one by one (and once more inside the struct): the hardware preloads the first 14 dwords
// of a kernel's arguments into scalar registers when it starts a wave (-amdgpu-kernarg-preload-count), but not the
// members of a struct passed by value.  What the kernel needs before its first requests then costs no load:
// 0.5 us less from the start of a workgroup to its first weight request.
__global__ void __launch_bounds__(512) k_skinny16(const uint4* Wp_, const uint4* Xp_, const float* ssq_in_, float* h_,
                                                  const float* gain_next_, int N_, int K_, int n_rows_, int s_pad_,
                                                  int ssq_parts_, int n_units, SkinnyArgs a_rest) {
  SkinnyArgs a = a_rest;
  a.Wp = Wp_; a.Xp = Xp_; a.ssq_in = ssq_in_; a.h = h_; a.gain_next = gain_next_;
  a.N = N_; a.K = K_; a.n_rows = n_rows_; a.s_pad = s_pad_; a.ssq_parts = ssq_parts_;
  // the 8 partial results meet in LDS CH tiles at a time: [8 waves][CH * TG][64 lanes] float4 <= 128 KiB
  constexpr int CH = (NT * TG > 16) ? 16 / TG : NT;
  static_assert(NT % CH == 0 && (MODE != SKM_SWIGLU || CH % 2 == 0), "tile chunking");
  constexpr int RS = (CH * TG * 64 + 511) / 512;   // output slots per thread and chunk
  extern __shared__ float4 red[];
  __shared__ float s_part[512];
  constexpr int TS = 4 / TG;        // workgroups per (tile unit, token block)
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int KS = a.K >> 5;
  // block id -> (unit, token block, token split).  Ids are dealt round-robin to the 8 XCDs; the workgroups
  // that read the same weight tiles (all token blocks and splits of a unit) sit 8 ids apart, so they run on
  // one XCD at about the same time and the tiles come from HBM once.
  const int nblk = (a.n_rows + 63) >> 6;
  const int j = blockIdx.x >> 3, inner = j % (TS * nblk);
  const int unit = (j / (TS * nblk)) * 8 + (blockIdx.x & 7);
  const int tb = inner / TS;
  const int tg0 = (inner % TS) * TG;
  if (unit >= n_units) return;
  const int tile0 = unit * NT;
  f32x4 acc[NT][TG];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int g = 0; g < TG; ++g) acc[t][g] = f32x4{0.f, 0.f, 0.f, 0.f};
  float sq[kSsqPerThread];
  if (MODE != SKM_RESID) ssq_issue(a.ssq_in, a.ssq_parts, a.s_pad, tb * 64, sq);
  // RESID, single chunk: this thread's residual / gain operands are requested up front
  float4 h_old[RS], g_next[RS];
  if (MODE == SKM_RESID && CH == NT) {
#pragma unroll
    for (int i = 0; i < RS; ++i) {
      const int slot = tid + 512 * i;
      h_old[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      g_next[i] = h_old[i];
      if (slot < NT * TG * 64) {
        const int t = slot / (TG * 64), g = (slot >> 6) % TG, l = slot & 63;
        const int tok = tb * 64 + (tg0 + g) * 16 + (l & 15);
        const int f0 = (tile0 + t) * 16 + (l >> 4) * 4;
        if (tok < a.n_rows) {
          h_old[i] = *(const float4*)(a.h + (size_t)tok * a.N + f0);
          g_next[i] = *(const float4*)(a.gain_next + f0);
        }
      }
    }
  }

  const uint4* wbase = a.Wp + (size_t)tile0 * KS * 64 + lane;
  const uint4* xbase = a.Xp + ((size_t)tb * KS * 4 + tg0) * 64 + lane;
  for (int k0 = wave; k0 < KS; k0 += 8 * R) {
    Frag16 wf[R][NT], xf[R][TG];
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int ks = k0 + 8 * i;
      if (ks < KS) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
          wf[i][t].n = __builtin_nontemporal_load((const u32x4*)(wbase + ((size_t)t * KS + ks) * 64));
#pragma unroll
        for (int g = 0; g < TG; ++g) xf[i][g].u = xbase[(size_t)(ks * 4 + g) * 64];
      }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int ks = k0 + 8 * i;
      if (ks < KS) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int g = 0; g < TG; ++g) acc[t][g] = mfma16(wf[i][t], xf[i][g], acc[t][g]);
      }
    }
  }
  if (MODE != SKM_RESID) ssq_publish(sq, a.ssq_parts, s_part);
  auto sum8 = [&](int tg, int l) -> float4 {   // tg = (t - chunk start) * TG + g
    float4 s = red[(size_t)tg * 64 + l];
#pragma unroll
    for (int w = 1; w < 8; ++w) {
      const float4 p = red[(size_t)(w * CH * TG + tg) * 64 + l];
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    return s;
  };
#pragma unroll
  for (int c0 = 0; c0 < NT; c0 += CH) {
    // cross-wave reduction of tiles c0 .. c0 + CH - 1
    if (c0 > 0) __syncthreads();
#pragma unroll
    for (int t = 0; t < CH; ++t)
#pragma unroll
      for (int g = 0; g < TG; ++g)
        red[(size_t)(wave * CH * TG + t * TG + g) * 64 + lane] =
            make_float4(acc[c0 + t][g][0], acc[c0 + t][g][1], acc[c0 + t][g][2], acc[c0 + t][g][3]);
    __syncthreads();
    if (MODE == SKM_SWIGLU) {
      const int KSo = (a.N >> 1) >> 5;   // act has F = N / 2 features
      for (int slot = tid; slot < (CH / 2) * TG * 64; slot += 512) {
        const int pp = slot / (TG * 64), g = (slot >> 6) % TG, l = slot & 63;
        const float4 gs = sum8((2 * pp) * TG + g, l), us = sum8((2 * pp + 1) * TG + g, l);
        const int tl = (tg0 + g) * 16 + (l & 15), tok = tb * 64 + tl;
        const int f0 = (((tile0 + c0) >> 1) + pp) * 16 + (l >> 4) * 4;
        f16x4 o;
        if (tok < a.n_rows) {
          const float sc = ssq_scale(s_part, tl, a.norm_dim, a.eps);
          o[0] = from_f32<f16>(silu_f(gs.x * sc) * (us.x * sc)); o[1] = from_f32<f16>(silu_f(gs.y * sc) * (us.y * sc));
          o[2] = from_f32<f16>(silu_f(gs.z * sc) * (us.z * sc)); o[3] = from_f32<f16>(silu_f(gs.w * sc) * (us.w * sc));
        } else {
          o[0] = o[1] = o[2] = o[3] = (f16)0.f;
        }
        *(f16x4*)((f16*)a.xp_out + x16_chunk(tok, f0, KSo) * 8 + (f0 & 4)) = o;
      }
    } else if (MODE == SKM_STORE) {
      for (int slot = tid; slot < CH * TG * 64; slot += 512) {
        const int t = slot / (TG * 64), g = (slot >> 6) % TG, l = slot & 63;
        const float4 s = sum8(t * TG + g, l);
        const int tl = (tg0 + g) * 16 + (l & 15), tok = tb * 64 + tl;
        const int f0 = (tile0 + c0 + t) * 16 + (l >> 4) * 4;
        if (tok < a.n_rows) {
          const float sc = ssq_scale(s_part, tl, a.norm_dim, a.eps);
          float4 o = make_float4(s.x * sc, s.y * sc, s.z * sc, s.w * sc);
          if (a.bias) {
            const float4 bb = *(const float4*)(a.bias + f0);
            o.x += bb.x; o.y += bb.y; o.z += bb.z; o.w += bb.w;
          }
          *(float4*)(a.out_f32 + (size_t)tok * a.ldc + f0) = o;
        }
      }
    } else {
      if (CH == NT) {
        // The operands requested up front are taken here, outside the branch on the row bound: otherwise the
        // compiler, which cannot see that they landed rounds ago, waits for every outstanding memory operation where
        // the branch rejoins - and that includes the residual store just issued, a full round trip in front of the
        // second store.
#pragma unroll
        for (int i = 0; i < RS; ++i)
          asm volatile("" ::"v"(h_old[i].x), "v"(h_old[i].y), "v"(h_old[i].z), "v"(h_old[i].w), "v"(g_next[i].x),
                       "v"(g_next[i].y), "v"(g_next[i].z), "v"(g_next[i].w));
      }
#pragma unroll
      for (int i = 0; i < RS; ++i) {
        const int slot = tid + 512 * i;
        if (slot >= CH * TG * 64) break;   // a whole wave leaves together (64 slots per wave)
        const int t = slot / (TG * 64), g = (slot >> 6) % TG, l = slot & 63;
        float4 s = sum8(t * TG + g, l);
        const int tok = tb * 64 + (tg0 + g) * 16 + (l & 15);
        const int f0 = (tile0 + c0 + t) * 16 + (l >> 4) * 4;
        f16x4 o;
        float q = 0.f;
        if (tok < a.n_rows) {
          float4 ho, gn;
          if (CH == NT) { ho = h_old[i]; gn = g_next[i]; }
          else { ho = *(const float4*)(a.h + (size_t)tok * a.N + f0); gn = *(const float4*)(a.gain_next + f0); }
          s.x += ho.x; s.y += ho.y; s.z += ho.z; s.w += ho.w;
          *(float4*)(a.h + (size_t)tok * a.N + f0) = s;
          o[0] = from_f32<f16>(s.x * gn.x); o[1] = from_f32<f16>(s.y * gn.y);
          o[2] = from_f32<f16>(s.z * gn.z); o[3] = from_f32<f16>(s.w * gn.w);
          q = s.x * s.x + s.y * s.y + s.z * s.z + s.w * s.w;
        } else {
          o[0] = o[1] = o[2] = o[3] = (f16)0.f;
        }
        *(f16x4*)((f16*)a.xp_out + x16_chunk(tok, f0, a.N >> 5) * 8 + (f0 & 4)) = o;
        q = sum_xor16(q);
        q = sum_xor32(q);
        if (l < 16) a.ssq_out[(size_t)(tile0 + c0 + t) * a.s_pad + tok] = q;
      }
    }
  }
}

template <int NT, int TG, int R, int MODE>
static hipError_t launch_skinny(const SkinnyArgs& a, hipStream_t st) {
  constexpr int CH = (NT * TG > 16) ? 16 / TG : NT;
  static bool attr_done = false;
  const size_t smem = (size_t)8 * CH * TG * 64 * sizeof(float4);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_skinny16<NT, TG, R, MODE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if ((a.N / 16) % NT != 0) return hipErrorInvalidValue;
  const int units = a.N / 16 / NT;
  const int blocks = (a.n_rows + 63) / 64;
  const int gx = (units + 7) / 8 * 8 * (4 / TG) * blocks;
  return launch(KID_GEMM_SKINNY, k_skinny16<NT, TG, R, MODE>, dim3(gx), dim3(512), smem, st, a.Wp, a.Xp, a.ssq_in, a.h, a.gain_next,
                a.N, a.K, a.n_rows, a.s_pad, a.ssq_parts, units, a);
}

// Blocking.  A workgroup reads NT weight tiles and TG token groups over the whole K, so what it must
// ingest is (NT + TG) * K * 32 bytes for NT * TG output tiles.  With one 64-token block the kernels
// are latency-bound and small workgroups win (1 x 1; the gate/up pairs 4 x 4); with several blocks
// the re-reads of the token operand dominate and the blocking goes towards square.
hipError_t d_gemm_skinny(const SkinnyArgs& a, int mode, hipStream_t st) {
  if (a.K % 32 != 0 || a.N % 16 != 0 || a.n_rows <= 0) return hipErrorInvalidValue;
  if (mode != SKM_RESID && (a.ssq_in == nullptr || a.ssq_parts < 1 || a.ssq_parts > 8 * kSsqPerThread)) return hipErrorInvalidValue;
  const int per_wave = ((a.K >> 5) + 7) / 8;   // k steps per wave
  const int tiles = a.N / 16;
  const bool multi = a.n_rows > 64;
  if (mode == SKM_SWIGLU) {
    if (a.N % 64 != 0) return hipErrorInvalidValue;
    if (multi && tiles % 8 == 0) return launch_skinny<8, 4, 2, SKM_SWIGLU>(a, st);
    if (per_wave <= 4) return launch_skinny<4, 4, 4, SKM_SWIGLU>(a, st);
    return launch_skinny<2, 4, 6, SKM_SWIGLU>(a, st);
  }
  // several token blocks and a narrow output: 4 x 4 blocking would leave compute units idle (1.5B QKV at 256 rows:
  // 128 workgroups of 393 KB); two tiles per workgroup double the workgroups at 295 KB each
  const bool few = multi && tiles % 4 == 0 && (tiles / 4) * ((a.n_rows + 63) / 64) < 192;
  // one token block, more 16-token workgroups than compute units (0.5B QKV: 72 tiles x 4 = 288): some compute
  // units would get two workgroups and ingest twice; 32-token workgroups (144 of them, 86 KB each) keep it one each
  const bool tg2 = !multi && tiles * 4 > 256;
  if (mode == SKM_STORE) {
    if (few) return launch_skinny<2, 4, 3, SKM_STORE>(a, st);
    if (multi && tiles % 4 == 0) return launch_skinny<4, 4, 3, SKM_STORE>(a, st);
    if (tg2) return per_wave <= 4 ? launch_skinny<1, 2, 4, SKM_STORE>(a, st) : launch_skinny<1, 2, 8, SKM_STORE>(a, st);
    if (per_wave <= 4) return launch_skinny<1, 1, 4, SKM_STORE>(a, st);
    return launch_skinny<1, 1, 8, SKM_STORE>(a, st);
  }
  if (few && per_wave <= 8) return launch_skinny<2, 4, 3, SKM_RESID>(a, st);
  if (multi && per_wave <= 8 && tiles % 4 == 0) return launch_skinny<4, 4, 3, SKM_RESID>(a, st);
  if (multi && tiles % 2 == 0) return launch_skinny<2, 2, 9, SKM_RESID>(a, st);
  if (tg2 && per_wave <= 4) return launch_skinny<1, 2, 4, SKM_RESID>(a, st);
  if (tg2 && per_wave <= 8) return launch_skinny<1, 2, 8, SKM_RESID>(a, st);
  if (per_wave <= 4) return launch_skinny<1, 1, 4, SKM_RESID>(a, st);
  if (per_wave <= 8) return launch_skinny<1, 1, 8, SKM_RESID>(a, st);
  return launch_skinny<1, 1, 20, SKM_RESID>(a, st);
}

// ---------------------------------------------------------------------------------------
// Rows of the residual stream -> X16 order: xp = half(h * gain), ssq[row] = sum h^2 (one part).
// One workgroup of 128 threads per row; thread i handles the 8 features 8 i .. 8 i + 7 (+1024 j).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void row_to_x16(const float (&v)[8], const float* __restrict__ gain, int k, int row, int KS,
                                           uint4* __restrict__ xp) {
  Frag16 f;
#pragma unroll
  for (int e = 0; e < 8; ++e) f.h[e] = from_f32<f16>(v[e] * gain[k + e]);
  xp[x16_chunk(row, k, KS)] = f.u;
}
__device__ __forceinline__ float block128_sum(float s, float* red) {
  s = wave_reduce_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  return red[0] + red[1];
}

__global__ void __launch_bounds__(128) k_pack_rows_x16(const float* __restrict__ h, const float* __restrict__ gain, int d,
                                                       uint4* __restrict__ xp, float* __restrict__ ssq) {
  __shared__ float red[2];
  const int row = blockIdx.x;
  float ss = 0.f;
  for (int k = threadIdx.x * 8; k < d; k += 1024) {
    float v[8];
    const float4 a = *(const float4*)(h + (size_t)row * d + k), b = *(const float4*)(h + (size_t)row * d + k + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
    row_to_x16(v, gain, k, row, d >> 5, xp);
  }
  ss = block128_sum(ss, red);
  if (threadIdx.x == 0) ssq[row] = ss;
}
hipError_t d_pack_rows_x16(const float* h, const float* gain, int M, int d, void* xp, float* ssq, hipStream_t st) {
  return launch(KID_MISC, k_pack_rows_x16, dim3(M), dim3(128), 0, st, h, gain, d, (uint4*)xp, ssq);
}

// The same after a split-K GEMM: h[row] += sum over the splits of partial[z][row] (added in split order),
// then xp and the sums of squares of the updated row, one part per 1024 features: ssq[part][s_pad].
// One workgroup of 128 threads per (row, 1024 features).
__global__ void __launch_bounds__(128) k_resid_finish_x16(const float* __restrict__ partial, int splits, size_t split_stride,
                                                          float* __restrict__ h, const float* __restrict__ gain, int d,
                                                          int s_pad, uint4* __restrict__ xp, float* __restrict__ ssq) {
  __shared__ float red[2];
  const int row = blockIdx.x, k = blockIdx.y * 1024 + threadIdx.x * 8;
  float ss = 0.f;
  if (k < d) {
    float v[8];
    float* hp = h + (size_t)row * d + k;
    const float4 a = *(const float4*)hp, b = *(const float4*)(hp + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
#pragma unroll 4
    for (int z = 0; z < splits; ++z) {
      const float* pp = partial + (size_t)z * split_stride + (size_t)row * d + k;
      const float4 pa = *(const float4*)pp, pb = *(const float4*)(pp + 4);
      v[0] += pa.x; v[1] += pa.y; v[2] += pa.z; v[3] += pa.w; v[4] += pb.x; v[5] += pb.y; v[6] += pb.z; v[7] += pb.w;
    }
    *(float4*)hp = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(hp + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
    row_to_x16(v, gain, k, row, d >> 5, xp);
  }
  ss = block128_sum(ss, red);
  if (threadIdx.x == 0) ssq[(size_t)blockIdx.y * s_pad + row] = ss;
}
hipError_t d_resid_finish_x16(const float* partial, int splits, size_t split_stride, float* h, const float* gain, int M, int d,
                              int s_pad, void* xp, float* ssq, hipStream_t st) {
  return launch(KID_MISC, k_resid_finish_x16, dim3(M, (d + 1023) / 1024), dim3(128), 0, st, partial, splits, split_stride, h,
                gain, d, s_pad, (uint4*)xp, ssq);
}

// Embedding row of token id `tok` -> h[row] (fp32), X16 half(h * gain), ssq[row].  128 threads.
__device__ __forceinline__ void embed_row_x16(const bf16* __restrict__ embed, int tok, int row, int d,
                                              const float* __restrict__ gain, float* __restrict__ h,
                                              uint4* __restrict__ xp, float* __restrict__ ssq, float* red) {
  float ss = 0.f;
  for (int k = threadIdx.x * 8; k < d; k += 1024) {
    Frag16 e; e.u = *(const uint4*)(embed + (size_t)tok * d + k);
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { v[i] = (float)e.v[i]; ss += v[i] * v[i]; }
    *(float4*)(h + (size_t)row * d + k) = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(h + (size_t)row * d + k + 4) = make_float4(v[4], v[5], v[6], v[7]);
    row_to_x16(v, gain, k, row, d >> 5, xp);
  }
  ss = block128_sum(ss, red);
  if (threadIdx.x == 0) ssq[row] = ss;
}

// Decode-side embedding gather of the token sampled at the previous step.
__global__ void __launch_bounds__(128) k_embed_x16(const int32_t* __restrict__ tokens, int tok_stride, const int* step,
                                                   const bf16* __restrict__ embed, int d, const float* __restrict__ gain,
                                                   float* __restrict__ h, uint4* __restrict__ xp, float* __restrict__ ssq,
                                                   const int* __restrict__ slot_seq) {
  __shared__ float red[2];
  const int row = blockIdx.x;
  const int seq = slot_seq ? slot_seq[row] : row;
  int tok = tokens[(size_t)seq * tok_stride + (*step - 1)];
  if (tok < 0) tok = 0;   // a step that reported a fault left -1 behind: never an index
  embed_row_x16(embed, tok, row, d, gain, h, xp, ssq, red);
}
hipError_t d_embed_x16(const int32_t* tokens, int tok_stride, const int* step, const void* embed, int M, int d,
                       const float* gain, float* h, void* xp, float* ssq, const int* slot_seq, hipStream_t st) {
  return launch(KID_EMBED, k_embed_x16, dim3(M), dim3(128), 0, st, tokens, tok_stride, step, (const bf16*)embed, d, gain, h,
                (uint4*)xp, ssq, slot_seq);
}

// ---------------------------------------------------------------------------------------
// LM head for decode: logits tile -> online log-sum-exp + Gumbel-max; logits are never stored.
// 512 threads = 8 waves; X (64 tokens x K, X16 order) is staged once into LDS and every wave owns
// whole 16-vocabulary tiles over the full K: tile = global wave index + j * (number of waves), its
// weights streamed in groups of U k steps with the next group in flight while the current one is
// multiplied.  A lane keeps, for its token of each 16-token group, the running (max, sum exp) and
// the best perturbed score; lanes, waves and workgroups are merged in a fixed order.
// partials: [n_wg][64][5] (max, sum exp, best y, its logit, its id).
// ---------------------------------------------------------------------------------------
struct LaneState {
  float m[4], l[4], by[4], bz[4];
  int bid[4];
};

// global -> LDS copy of one wave-wide 1 KiB block (lane l's 16 bytes land at lds + 16 l); completion is awaited with
// wait_vmcnt_d (requests complete in order)
__device__ __forceinline__ unsigned lds_addr16(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}
__device__ __forceinline__ void dma16_lds(const void* g, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt_d() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int U>
__global__ void __launch_bounds__(512) k_lmhead_sample16(const uint4* __restrict__ Wp, const uint4* __restrict__ Xp, int KS,
                                                         int n_tiles, const float* __restrict__ ssq, int ssq_parts,
                                                         int s_pad, int norm_dim, float eps, int n_rows, int seq0,
                                                         SampleParams sp, float* __restrict__ partials) {
  extern __shared__ uint4 xs[];   // [KS][4][64]
  __shared__ float s_part[512];
  __shared__ float s_scale[64];
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  // The wave's first weight group is requested before anything else, and the token operand goes to LDS without
  // passing through registers (copied through registers, every 16 bytes were one load, wait, LDS store - a
  // dependent round trip per loop pass, KS / 2 of them in front of the first weight request).
  int tile = blockIdx.x * 8 + wave;
  Frag16 cur[U], nxt[U];
  if (tile < n_tiles) {
    const uint4* wb = Wp + (size_t)tile * KS * 64 + lane;
#pragma unroll
    for (int i = 0; i < U; ++i) cur[i].n = __builtin_nontemporal_load((const u32x4*)(wb + (size_t)i * 64));
  }
  float sq[kSsqPerThread];
  ssq_issue(ssq, ssq_parts, s_pad, 0, sq);
  // the sampling parameters too (behind the copy below they would be read through the vector path, one more round trip)
  resolve_sample_params(sp);
  const int step = *sp.step;
  const bool noisy = sp.temperature != 0.f;
  const float inv_t = noisy ? 1.0f / sp.temperature : 1.0f;
  const int fq = lane >> 4, tl = lane & 15;
  uint32_t seq_id[4];   // the noise is keyed on the sequence, which need not be the row
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int row = g * 16 + tl;
    seq_id[g] = (uint32_t)((sp.slot_seq && row < n_rows) ? sp.slot_seq[row] : seq0 + row);
  }
  {
    const unsigned xs0 = __builtin_amdgcn_readfirstlane(lds_addr16(xs));
    for (int b = wave * 64; b < KS * 256; b += 512) dma16_lds(Xp + b + lane, xs0 + (unsigned)b * 16u);
  }
  ssq_publish(sq, ssq_parts, s_part);
  wait_vmcnt_d<0>();   // this wave's blocks of the operand have landed ...
  __syncthreads();     // ... and everybody's
  if (tid < 64) s_scale[tid] = ssq_scale(s_part, tid, norm_dim, eps);
  __syncthreads();
  float scale[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) scale[g] = s_scale[g * 16 + tl];
  LaneState stt;
#pragma unroll
  for (int g = 0; g < 4; ++g) { stt.m[g] = -INFINITY; stt.l[g] = 0.f; stt.by[g] = -INFINITY; stt.bz[g] = 0.f; stt.bid[g] = 0x7fffffff; }

  const int n_waves = gridDim.x * 8;
  const int groups_per_tile = KS / U;
  f32x4 acc[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
  int grp = 0;
  while (tile < n_tiles) {
    // prefetch the next group (of this tile, or the first of the wave's next tile)
    int ntile = tile, ngrp = grp + 1;
    if (ngrp == groups_per_tile) { ngrp = 0; ntile = tile + n_waves; }
    if (ntile < n_tiles) {
      const uint4* wb = Wp + ((size_t)ntile * KS + (size_t)ngrp * U) * 64 + lane;
#pragma unroll
      for (int i = 0; i < U; ++i) nxt[i].n = __builtin_nontemporal_load((const u32x4*)(wb + (size_t)i * 64));
    }
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int ks = grp * U + i;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        Frag16 x; x.u = xs[(ks * 4 + g) * 64 + lane];
        acc[g] = mfma16(cur[i], x, acc[g]);
      }
    }
    if (grp == groups_per_tile - 1) {
      const int v0 = tile * 16 + fq * 4;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float z[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) z[j] = acc[g][j] * scale[g];
        const float mt = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
        const float mn = fmaxf(stt.m[g], mt);
        stt.l[g] = stt.l[g] * __expf(stt.m[g] - mn) + ((__expf(z[0] - mn) + __expf(z[1] - mn)) + (__expf(z[2] - mn) + __expf(z[3] - mn)));
        stt.m[g] = mn;
        float gn[4] = {0.f, 0.f, 0.f, 0.f};
        if (noisy) gumbel4(sp.seed_lo, sp.seed_hi, seq_id[g], (uint32_t)step, (uint32_t)(v0 >> 2), gn);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float y = noisy ? z[j] * inv_t + gn[j] : z[j];
          if (y > stt.by[g]) { stt.by[g] = y; stt.bz[g] = z[j]; stt.bid[g] = v0 + j; }   // ids ascend: ties keep the lower id
        }
        acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int i = 0; i < U; ++i) cur[i] = nxt[i];
    tile = ntile; grp = ngrp;
  }
  // merge the 4 lanes that share a token (fixed order), then the 8 waves, one row of partials per token
  __syncthreads();          // everybody is done reading xs: reuse it
  float* sm = (float*)xs;   // [8 waves][64 tokens][5]
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    LseAcc a; a.m = stt.m[g]; a.l = stt.l[g];
    BestAcc b; b.y = stt.by[g]; b.z = stt.bz[g]; b.id = stt.bid[g];
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      a.merge(__shfl_xor(a.m, o, 64), __shfl_xor(a.l, o, 64));
      b.add(__shfl_xor(b.y, o, 64), __shfl_xor(b.z, o, 64), __shfl_xor(b.id, o, 64));
    }
    if (fq == 0) {
      float* p = sm + ((size_t)wave * 64 + g * 16 + tl) * 5;
      p[0] = a.m; p[1] = a.l; p[2] = b.y; p[3] = b.z; ((int*)p)[4] = b.id;
    }
  }
  __syncthreads();
  if (tid < 64) {
    LseAcc a; a.init();
    BestAcc b; b.init();
    for (int w = 0; w < 8; ++w) {
      const float* p = sm + ((size_t)w * 64 + tid) * 5;
      a.merge(p[0], p[1]);
      b.add(p[2], p[3], ((const int*)p)[4]);
    }
    float* p = partials + ((size_t)blockIdx.x * 64 + tid) * 5;
    p[0] = a.m; p[1] = a.l; p[2] = b.y; p[3] = b.z; ((int*)p)[4] = b.id;
  }
}

// Merge the per-workgroup partials of one sequence, write its token and log-prob, and gather the
// token's embedding row as the input of the next decode step (residual row, X16 row for the first
// layer's norm gain, sum of squares).  One workgroup of 128 threads per sequence.
__global__ void __launch_bounds__(128) k_lmhead_merge_embed(const float* __restrict__ partials, int n_wg, int row_stride,
                                                            int seq0, SampleParams sp, const bf16* __restrict__ embed, int d,
                                                            const float* __restrict__ gain, float* __restrict__ h,
                                                            uint4* __restrict__ xp, float* __restrict__ ssq) {
  __shared__ float red[2];
  __shared__ int s_tok;
  const int r = blockIdx.x, lane = threadIdx.x & 63;
  if (threadIdx.x < 64) {
    LseAcc a; a.init();
    BestAcc b; b.init();
    for (int w = lane; w < n_wg; w += 64) {
      const float* p = partials + ((size_t)w * row_stride + r) * 5;
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
      s_tok = emit_token(sp, sp.slot_seq ? sp.slot_seq[r] : seq0 + r, step, b.id, b.z - (a.m + logf(a.l)));
      // every workgroup has used the step index before it arrives here: the last one to arrive moves it on
      if (sp.arrivals && atomicAdd(sp.arrivals, 1) == (int)gridDim.x - 1) {
        *sp.arrivals = 0;
        *const_cast<int*>(sp.step) = step + 1;
      }
    }
  }
  __syncthreads();
  embed_row_x16(embed, s_tok, seq0 + r, d, gain, h, xp, ssq, red);
}

size_t d_lmhead_sample_partial_floats() { return (size_t)256 * 64 * 5; }

template <int U>
static hipError_t launch_lmhead(const uint4* Wp, const uint4* Xp, int KS, int n_tiles, const float* ssq, int ssq_parts,
                                int s_pad, int norm_dim, float eps, int n_rows, int seq0, SampleParams sp, float* partials,
                                int n_wg, hipStream_t st) {
  static bool attr_done = false;
  const size_t smem = (size_t)KS * 256 * sizeof(uint4) < 8 * 64 * 5 * 4 ? 8 * 64 * 5 * 4 : (size_t)KS * 256 * sizeof(uint4);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_lmhead_sample16<U>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  return launch(KID_LMHEAD_SAMPLE, k_lmhead_sample16<U>, dim3(n_wg), dim3(512), smem, st, Wp, Xp, KS, n_tiles, ssq, ssq_parts, s_pad, norm_dim, eps, n_rows, seq0, sp,
                                                partials);
}

bool d_lmhead_sample_supported(int K, int n_rows) { return n_rows <= 64 && K % 32 == 0 && (size_t)K * 128 <= 131072; }

hipError_t d_lmhead_sample(const void* Wp, const void* Xp, int K, int V, const float* ssq, int ssq_parts, int s_pad,
                           float eps, int n_rows, SampleParams sp, float* partials, const void* embed,
                           const float* gain_first, float* h, void* xp_first, float* ssq_first, hipStream_t st) {
  if (!d_lmhead_sample_supported(K, n_rows) || V % 16 != 0 || ssq == nullptr || ssq_parts < 1 || ssq_parts > 8 * kSsqPerThread)
    return hipErrorInvalidValue;
  const int KS = K / 32, n_tiles = V / 16;
  int n_wg = 256;
  if (n_wg > (n_tiles + 7) / 8) n_wg = (n_tiles + 7) / 8;
  hipError_t e;
  {
    if (KS % 7 == 0)
      e = launch_lmhead<7>((const uint4*)Wp, (const uint4*)Xp, KS, n_tiles, ssq, ssq_parts, s_pad, K, eps, n_rows, 0, sp, partials, n_wg, st);
    else if (KS % 4 == 0)
      e = launch_lmhead<4>((const uint4*)Wp, (const uint4*)Xp, KS, n_tiles, ssq, ssq_parts, s_pad, K, eps, n_rows, 0, sp, partials, n_wg, st);
    else
      e = launch_lmhead<1>((const uint4*)Wp, (const uint4*)Xp, KS, n_tiles, ssq, ssq_parts, s_pad, K, eps, n_rows, 0, sp, partials, n_wg, st);
  }
  if (e != hipSuccess) return e;
  return d_lmhead_merge_embed(partials, n_wg, 64, n_rows, sp, embed, K, gain_first, h, xp_first, ssq_first, st);
}

hipError_t d_lmhead_merge_embed(const float* partials, int n_parts, int row_stride, int n_rows, SampleParams sp,
                                const void* embed, int d, const float* gain_first, float* h, void* xp_first,
                                float* ssq_first, hipStream_t st) {
  return launch(KID_LMHEAD_SAMPLE_MERGE, k_lmhead_merge_embed, dim3(n_rows), dim3(128), 0, st, partials, n_parts, row_stride,
                0, sp, (const bf16*)embed, d, gain_first, h, (uint4*)xp_first, ssq_first);
}

// =======================================================================================
// Decode attention over the paged KV cache, fused with rotary + KV append of the new token.
// One workgroup (NW waves) per (sequence, KV head); all query heads of the group ride together as
// the 16 columns of 16x16x32 MFMAs.  S^T = K Q^T (tokens x queries) so that each lane owns one
// query column: the running max / sum are per-lane scalars plus two cross-lane shuffles, and the
// probabilities a lane produces are exactly its operand of O^T = V^T P^T.  Token rows are permuted
// inside a 32-token page pair so that a lane's 8 probabilities are 8 consecutive tokens, which is
// what the token-minor V page delivers in one 16-byte load.  Waves take page pairs round-robin, PD
// pairs at a time with all their K/V fragments in flight at once; the first chunk is requested
// before the query rows are even read (K/V addresses depend on the page table only), so a step
// pays one memory round trip, not one per dependent stage.  Waves are merged through LDS.
// Queries, keys, values and probabilities are IEEE half (the cache's type on this path); the
// output goes out as half in X16 order (the O projection's operand).
// ---------------------------------------------------------------------------------------
// The prefix workgroup of the shared-prompt variant (see ShareArgs): block (prompt p, KV head kvh) walks the page
// pairs 0 .. prefix_pairs - 1 of the prompt once, with the query heads of all G siblings as columns of up to four
// 16-column MFMA tiles (column c = sibling c / rep, head c % rep), and leaves per column the merged, unnormalised
// (max, sum, weighted values) of its waves in sh.pre, stored write-through; then it publishes the launch number.
template <int HD, int NW>
__device__ __forceinline__ void attention_prefix_role(const float* __restrict__ qkv, const float2* __restrict__ rope,
                                                      const RowMap& rm, const KVCache& kv, int n_q_heads,
                                                      const ShareArgs& sh, float* sm_o, f16* qs64, float (*sm_m)[16],
                                                      float (*sm_l)[16]) {
  constexpr int KK = HD / 32, DT = HD / 16, NT = kSharePrefixMaxColumns / 16;
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int qcol = lane & 15, grp = lane >> 4;
  const int hkv = kv.n_kv_heads, rep = n_q_heads / hkv;
  const int p = blockIdx.x / hkv, kvh = blockIdx.x % hkv;
  const int row0 = p * sh.G;
  const int ncols = sh.G * rep;
  int seq, pos;
  rm.get(row0, seq, pos);             // every sibling is at this position; the shared pages are the same for all
  const int* pt = kv.page_table + (size_t)seq * kv.pages_per_seq;
  const f16* kpool = (const f16*)kv.k;
  const f16* vpool = (const f16*)kv.v;
  const size_t page_elems = (size_t)hkv * kPageTokens * HD;
  auto load_pair = [&](int pp, Frag16 (&kf)[2][KK], Frag16 (&vf)[DT]) {
    const int pa = pt[2 * pp], pb = pt[2 * pp + 1];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = lane & 15;
      const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);
      const f16* kp = kpool + (size_t)(ptok < 16 ? pa : pb) * page_elems + ((size_t)kvh * kPageTokens + (ptok & 15)) * HD;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[t][kk].u = *(const uint4*)(kp + kk * 32 + grp * 8);
    }
    const f16* vp = vpool + (size_t)(grp < 2 ? pa : pb) * page_elems + (size_t)kvh * HD * kPageTokens + (grp & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[dt].u = *(const uint4*)(vp + (size_t)(dt * 16 + (lane & 15)) * kPageTokens);
  };
  Frag16 kf[2][2][KK], vf[2][DT];
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (wave + NW * j < sh.prefix_pairs) load_pair(wave + NW * j, kf[j], vf[j]);
  // rotated queries of every column (zero rows for the columns past G x rep)
  {
    const int half = HD / 2;
    const size_t row_floats = (size_t)(n_q_heads + 2 * hkv) * HD;
    for (int idx = tid; idx < NT * 16 * half; idx += NW * 64) {
      const int cc = idx / half, i = idx % half;
      float r1 = 0.f, r2 = 0.f;
      if (cc < ncols) {
        const float* x = qkv + (size_t)(row0 + cc / rep) * row_floats + (size_t)(kvh * rep + cc % rep) * HD;
        const float2 cs = rope[(size_t)pos * half + i];
        r1 = rot_first(x[i], x[i + half], cs.x, cs.y);
        r2 = rot_second(x[i], x[i + half], cs.x, cs.y);
      }
      qs64[cc * HD + i] = from_f32<f16>(r1);
      qs64[cc * HD + i + half] = from_f32<f16>(r2);
    }
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)HD);
  float m_run[NT], l_run[NT];
  f32x4 o[NT][DT];
#pragma unroll
  for (int jt = 0; jt < NT; ++jt) {
    m_run[jt] = -INFINITY; l_run[jt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[jt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  for (int c0 = 0; wave + NW * c0 < sh.prefix_pairs; c0 += 2) {
    if (c0 > 0) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (wave + NW * (c0 + j) < sh.prefix_pairs) load_pair(wave + NW * (c0 + j), kf[j], vf[j]);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (wave + NW * (c0 + j) >= sh.prefix_pairs) break;
#pragma unroll
      for (int jt = 0; jt < NT; ++jt) {
        Frag16 qf[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk].u = *(const uint4*)(qs64 + (jt * 16 + qcol) * HD + kk * 32 + grp * 8);
        f32x4 sc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) sc[t] = mfma16(kf[j][t][kk], qf[kk], sc[t]);
        }
        // every token of a shared pair lies inside every sibling's context: nothing to mask
        float pv[8];
        float m_loc = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          pv[e] = sc[e >> 2][e & 3] * scale;
          m_loc = fmaxf(m_loc, pv[e]);
        }
        m_loc = max_xor16(m_loc);
        m_loc = max_xor32(m_loc);
        const float m_new = fmaxf(m_run[jt], m_loc);
        const float alpha = __expf(m_run[jt] - m_new);
        float psum = 0.f;
        Frag16 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = __expf(pv[e] - m_new);
          psum += pe;
          pf.h[e] = (f16)pe;
        }
        l_run[jt] = l_run[jt] * alpha + psum;
        m_run[jt] = m_new;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
          for (int i = 0; i < 4; ++i) o[jt][dt][i] *= alpha;
          o[jt][dt] = mfma16(vf[j][dt], pf, o[jt][dt]);
        }
      }
    }
  }
  // merge the waves tile by tile; a wave without a pair carries (-inf, 0, 0) and drops out (wave 0 always has pair 0)
#pragma unroll
  for (int jt = 0; jt < NT; ++jt) {
    float l = l_run[jt];
    l = sum_xor16(l);
    l = sum_xor32(l);
    if (jt > 0) __syncthreads();   // the previous tile's sums have been read
    if (grp == 0) { sm_m[wave][qcol] = m_run[jt]; sm_l[wave][qcol] = l; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) sm_o[((size_t)wave * HD + dt * 16 + grp * 4 + i) * 16 + qcol] = o[jt][dt][i];
    __syncthreads();
    for (int idx = tid; idx < 16 * (HD / 8); idx += NW * 64) {
      const int q = idx / (HD / 8), d0 = (idx % (HD / 8)) * 8;
      const int cc = jt * 16 + q;
      if (cc >= ncols) continue;
      float mx = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; ++w) mx = fmaxf(mx, sm_m[w][q]);
      float den = 0.f, wgt[NW];
#pragma unroll
      for (int w = 0; w < NW; ++w) { wgt[w] = __expf(sm_m[w][q] - mx); den += wgt[w] * sm_l[w][q]; }
      float num[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        num[e] = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) num[e] += wgt[w] * sm_o[((size_t)w * HD + d0 + e) * 16 + q];
      }
      const size_t base = ((size_t)(row0 + cc / rep) * n_q_heads + kvh * rep + cc % rep) * (HD + 4);
      st_f4<true>(sh.pre, (base + 4 + d0) * sizeof(float), make_float4(num[0], num[1], num[2], num[3]));
      st_f4<true>(sh.pre, (base + 8 + d0) * sizeof(float), make_float4(num[4], num[5], num[6], num[7]));
      if (d0 == 0) {
        st_f32<true>(sh.pre, base * sizeof(float), mx);
        st_f32<true>(sh.pre, (base + 1) * sizeof(float), den);
      }
    }
  }
  coh_drain();        // this thread's write-through stores have completed ...
  __syncthreads();    // ... and everybody's
  if (tid == 0) {
    const unsigned launch_no = (unsigned)(*rm.step) * (unsigned)sh.n_layers + (unsigned)sh.layer + 1u;
    (void)__hip_atomic_exchange(&sh.flags[blockIdx.x], launch_no, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// LDS = true is the measured alternative to the register-direct K/V reads: the same requests go global -> LDS
// (one 1 KiB block per fragment, lane l's 16 bytes at 16 l, so the read back is conflict-free) into PD slots per
// wave and are read into registers pair by pair; the requests in flight and the order of the arithmetic are the
// same, the results bit-identical.
// SHARE = true: the shared-prompt variant (ShareArgs): the first sh.n_prefix blocks are prefix workgroups, the others
// cover page pairs sh.prefix_pairs .. of their row and fold the prefix workgroup's partial result into the merge.
template <int HD, int NW, int PD, bool LDS, bool SHARE>
__global__ void __launch_bounds__(NW * 64) k_decode_attention16(const float* __restrict__ qkv,
                                                               const float2* __restrict__ rope, const int* step_,
                                                               const int* page_table_, int Lp_, int pages_per_seq_,
                                                               int n_kv_heads_, int n_q_heads, void* kpool_, RowMap rm,
                                                               KVCache kv, uint4* __restrict__ out, ShareArgs sh) {
  // what leads from the start of the kernel to its first requests arrives preloaded (see k_skinny16): 14 dwords
  rm.step = step_; rm.Lp = Lp_;
  kv.page_table = page_table_; kv.pages_per_seq = pages_per_seq_; kv.n_kv_heads = n_kv_heads_; kv.k = kpool_;
  constexpr int KK = HD / 32;   // k steps of S^T = K Q^T
  constexpr int DT = HD / 16;   // 16-row tiles of O^T
  constexpr int NFRAG = 2 * KK + DT;                        // 1 KiB fragments of one page pair
  constexpr size_t kOStride = LDS ? (size_t)PD * NFRAG * 256 : (size_t)HD * 16;   // floats between two waves' outputs
  extern __shared__ float sm_o[];   // [NW][HD][16]; LDS: [NW][PD][NFRAG] KiB of staged pairs, a wave's output over its slot 0
  __shared__ __attribute__((aligned(16))) f16 qs[16 * HD];
  __shared__ __attribute__((aligned(16))) f16 knew[HD];
  __shared__ __attribute__((aligned(16))) f16 vnew[HD];
  __shared__ float sm_m[NW][16], sm_l[NW][16];
  if constexpr (SHARE) {
    static_assert(!LDS, "the shared-prompt variant reads K/V register-direct");
    if ((int)blockIdx.x < sh.n_prefix) {   // uniform over the workgroup
      attention_prefix_role<HD, NW>(qkv, rope, rm, kv, n_q_heads, sh, sm_o, (f16*)(sm_o + (size_t)NW * HD * 16), sm_m, sm_l);
      return;
    }
  }
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int qcol = lane & 15, grp = lane >> 4;
  const int hkv = kv.n_kv_heads, rep = n_q_heads / hkv;
  const int bid = SHARE ? (int)blockIdx.x - sh.n_prefix : (int)blockIdx.x;
  const int s = bid / hkv, kvh = bid % hkv;
  const int pp0 = SHARE ? sh.prefix_pairs : 0;   // first page pair this workgroup covers
  int seq, pos;
  rm.get(s, seq, pos);
  const int ctx = pos + 1;
  const int* pt = kv.page_table + (size_t)seq * kv.pages_per_seq;
  f16* kpool = (f16*)kv.k;
  f16* vpool = (f16*)kv.v;
  const size_t page_elems = (size_t)hkv * kPageTokens * HD;
  const int npairs = (ctx + 31) / 32;
  const int last_page = (ctx - 1) / kPageTokens;

  // K rows of the two score tiles and the V tile of page pair pp: tile t row r is pair-token
  // 8 (r / 4) + 4 t + r % 4; the lane's V chunk holds pair-tokens 8 grp .. 8 grp + 7
  auto load_pages = [&](int pa, int pb, Frag16 (&kf)[2][KK], Frag16 (&vf)[DT]) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = lane & 15;
      const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);
      const f16* kp = kpool + (size_t)(ptok < 16 ? pa : pb) * page_elems + ((size_t)kvh * kPageTokens + (ptok & 15)) * HD;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[t][kk].u = *(const uint4*)(kp + kk * 32 + grp * 8);
    }
    const f16* vp = vpool + (size_t)(grp < 2 ? pa : pb) * page_elems + (size_t)kvh * HD * kPageTokens + (grp & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[dt].u = *(const uint4*)(vp + (size_t)(dt * 16 + (lane & 15)) * kPageTokens);
  };
  auto load_pair = [&](int pp, Frag16 (&kf)[2][KK], Frag16 (&vf)[DT]) {
    load_pages(pt[2 * pp], pt[min(2 * pp + 1, last_page)], kf, vf);
  };
  // the same requests into slot j of this wave's staging area
  const unsigned stage0 = LDS ? __builtin_amdgcn_readfirstlane(lds_addr16(sm_o) + (unsigned)wave * PD * NFRAG * 1024u) : 0u;
  auto stage_pages = [&](int pa, int pb, int j) {
    const unsigned dst = stage0 + (unsigned)j * NFRAG * 1024u;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = lane & 15;
      const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);
      const f16* kp = kpool + (size_t)(ptok < 16 ? pa : pb) * page_elems + ((size_t)kvh * kPageTokens + (ptok & 15)) * HD;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) dma16_lds(kp + kk * 32 + grp * 8, dst + (unsigned)(t * KK + kk) * 1024u);
    }
    const f16* vp = vpool + (size_t)(grp < 2 ? pa : pb) * page_elems + (size_t)kvh * HD * kPageTokens + (grp & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) dma16_lds(vp + (size_t)(dt * 16 + (lane & 15)) * kPageTokens, dst + (unsigned)(2 * KK + dt) * 1024u);
  };
  auto stage_pair = [&](int pp, int j) { stage_pages(pt[2 * pp], pt[min(2 * pp + 1, last_page)], j); };
  auto read_pair = [&](int j, Frag16 (&kf)[2][KK], Frag16 (&vf)[DT]) {
    const uint4* src = (const uint4*)sm_o + ((size_t)(wave * PD + j) * NFRAG) * 64 + lane;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[t][kk].u = src[(t * KK + kk) * 64];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[dt].u = src[(2 * KK + dt) * 64];
  };
  // The row's own q / k / v values and rotary pairs are requested before the cached pages: loads complete in the
  // order they were issued, so behind the pages they would be waited for together with every page in flight, and
  // behind the appended key's stores together with those stores' acknowledgements.
  constexpr int half = HD / 2;
  constexpr int NQ = 16 * half / (NW * 64);   // query elements per thread
  static_assert(NQ * NW * 64 == 16 * half && half <= NW * 64 && HD <= NW * 64, "whole passes over the 16 query rows");
  const float* row = qkv + (size_t)s * (n_q_heads + 2 * hkv) * HD;
  const int new_page = pt[pos / kPageTokens], new_slot = pos % kPageTokens;
  // every thread asks (clamped to a valid row or element) so that nothing here sits under a branch
  float qx1[NQ], qx2[NQ];
  float2 qcs[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const int idx = tid + n * NW * 64, r = min(idx / half, rep - 1), i = idx % half;
    const float* x = row + (size_t)(kvh * rep + r) * HD;
    qx1[n] = x[i];
    qx2[n] = x[i + half];
  }
  const int ki = min(tid, half - 1), vi = min(tid, HD - 1);
  float kx1 = row[(size_t)(n_q_heads + kvh) * HD + ki], kx2 = row[(size_t)(n_q_heads + kvh) * HD + ki + half];
  float vx = row[(size_t)(n_q_heads + hkv + kvh) * HD + vi];
  // ... the rotary pairs behind them: they need the position, which is a load away (the step counter)
#pragma unroll
  for (int n = 0; n < NQ; ++n) qcs[n] = rope[(size_t)pos * half + (tid + n * NW * 64) % half];
  float2 kcs = rope[(size_t)pos * half + ki];
  __builtin_amdgcn_sched_barrier(0);   // ... and these requests stay in front of the pages'

  constexpr int PR = LDS ? 1 : PD;   // register sets of fragments
  Frag16 kf[PR][2][KK], vf[PR][DT];
  // ---- the first page pairs are requested; rotary on the group's queries and the new key; append key / value ----
  // The number of pairs a wave requests (0 .. PD, wave-uniform) selects one of PD + 1 copies of the code: within a
  // copy the compiler knows how many requests stand behind the row's own values and waits for those alone, while
  // the pages are still on their way.  (Requests under a branch each would leave it a wait for everything; asking
  // for a page again in place of a missing pair costs more than it saves: a compute unit's ingest is the bound.)
  int first_pa[PD], first_pb[PD];   // looked up here (a missing pair: the last one's entries, unused) rather than in the copies
#pragma unroll
  for (int j = 0; j < PD; ++j) {
    const int pp = min(pp0 + wave + NW * j, npairs - 1);
    first_pa[j] = pt[2 * pp];
    first_pb[j] = pt[min(2 * pp + 1, last_page)];
  }
  auto first_pairs_and_rotary = [&](auto n_c) {
    constexpr int n_req = decltype(n_c)::value;
#pragma unroll
    for (int j = 0; j < n_req; ++j) {
      if constexpr (LDS) stage_pages(first_pa[j], first_pb[j], j);
      else load_pages(first_pa[j], first_pb[j], kf[j], vf[j]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      const int idx = tid + n * NW * 64, r = idx / half, i = idx % half;
      const bool live = r < rep;   // columns past the group's heads are zero
      qs[r * HD + i] = from_f32<f16>(live ? rot_first(qx1[n], qx2[n], qcs[n].x, qcs[n].y) : 0.f);
      qs[r * HD + i + half] = from_f32<f16>(live ? rot_second(qx1[n], qx2[n], qcs[n].x, qcs[n].y) : 0.f);
    }
    if (tid < half) {
      f16* kp = kpool + (size_t)new_page * page_elems + ((size_t)kvh * kPageTokens + new_slot) * HD;
      const f16 k1 = from_f32<f16>(rot_first(kx1, kx2, kcs.x, kcs.y)), k2 = from_f32<f16>(rot_second(kx1, kx2, kcs.x, kcs.y));
      kp[tid] = k1; kp[tid + half] = k2;
      knew[tid] = k1; knew[tid + half] = k2;
    }
    if (tid < HD) {
      const f16 vv = from_f32<f16>(vx);
      vpool[(size_t)new_page * page_elems + ((size_t)kvh * HD + tid) * kPageTokens + new_slot] = vv;
      vnew[tid] = vv;
    }
  };
  {
    static_assert(PD <= 3, "one copy per number of requested pairs");
    const int mine = npairs - pp0 - wave;                                // pairs wave, wave + NW, ... below it
    const int n_req = mine <= 0 ? 0 : min((mine + NW - 1) / NW, PD);
    if (n_req == 0) first_pairs_and_rotary(std::integral_constant<int, 0>());
    else if (n_req == 1 || PD == 1) first_pairs_and_rotary(std::integral_constant<int, 1>());
    else if (n_req == 2 || PD == 2) first_pairs_and_rotary(std::integral_constant<int, (PD >= 2 ? 2 : 1)>());
    else first_pairs_and_rotary(std::integral_constant<int, PD>());
  }
  __syncthreads();
  Frag16 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk].u = *(const uint4*)(qs + qcol * HD + kk * 32 + grp * 8);
  const float scale = 1.0f / sqrtf((float)HD);
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int c0 = 0; pp0 + wave + NW * c0 < npairs; c0 += PD) {
    if (c0 > 0) {
#pragma unroll
      for (int j = 0; j < PD; ++j)
        if (pp0 + wave + NW * (c0 + j) < npairs) {
          if constexpr (LDS) stage_pair(pp0 + wave + NW * (c0 + j), j);   // every slot has been read into registers and used
          else load_pair(pp0 + wave + NW * (c0 + j), kf[j], vf[j]);
        }
    }
    // pairs of this chunk that exist for this wave (LDS: requests issued above, in slot order)
    const int n_chunk = min(PD, (npairs - (pp0 + wave + NW * c0) + NW - 1) / NW);
#pragma unroll
    for (int jj = 0; jj < PD; ++jj) {
      const int pp = pp0 + wave + NW * (c0 + jj);
      if (pp >= npairs) break;
      constexpr int kSetStride = LDS ? 0 : 1;
      const int j = jj * kSetStride;          // register set: the pair's own, or the single one of the LDS variant
      if constexpr (LDS) {
        // slot jj has landed once at most the later slots' requests are outstanding (requests complete in order)
        const int newer = n_chunk - 1 - jj;
        if (newer >= 3) wait_vmcnt_d<3 * NFRAG>();
        else if (newer == 2) wait_vmcnt_d<2 * NFRAG>();
        else if (newer == 1) wait_vmcnt_d<NFRAG>();
        else wait_vmcnt_d<0>();
        asm volatile("" ::: "memory");
        read_pair(jj, kf[0], vf[0]);
      }
      // the token appended by this workgroup comes from LDS, not from the global copy written above
      if (pp == pos / 32) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int r = lane & 15;
          const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);
          if (ptok == pos % 32) {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kf[j][t][kk].u = *(const uint4*)(knew + kk * 32 + grp * 8);
          }
        }
        if (grp == (pos % 32) / 8) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) vf[j][dt].h[pos % 8] = vnew[dt * 16 + (lane & 15)];
        }
      }
      f32x4 sc[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) sc[t] = mfma16(kf[j][t][kk], qf[kk], sc[t]);
      }
      // lane (query qcol, group grp) now holds pair-tokens 8 grp + e, e = 4 t + i
      float p[8];
      float m_loc = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int n = pp * 32 + 8 * grp + e;
        const float sv = sc[e >> 2][e & 3] * scale;
        p[e] = (n < ctx) ? sv : -INFINITY;
        m_loc = fmaxf(m_loc, p[e]);
      }
      m_loc = max_xor16(m_loc);
      m_loc = max_xor32(m_loc);
      const float m_new = fmaxf(m_run, m_loc);
      const float alpha = __expf(m_run - m_new);
      float psum = 0.f;
      Frag16 pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = __expf(p[e] - m_new);
        psum += pe;
        pf.h[e] = (f16)pe;
      }
      l_run = l_run * alpha + psum;
      m_run = m_new;
      // tokens past the context may hold anything in V (even NaN bit patterns): zero them
      {
        const int nvalid = ctx - (pp * 32 + 8 * grp);   // lane's 8 tokens: first nvalid are real
        if (nvalid < 8) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (e >= nvalid) vf[j][dt].h[e] = (f16)0.f;
        }
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[dt][i] *= alpha;
        o[dt] = mfma16(vf[j][dt], pf, o[dt]);
      }
    }
  }
  l_run = sum_xor16(l_run);
  l_run = sum_xor32(l_run);
  if (grp == 0) { sm_m[wave][qcol] = m_run; sm_l[wave][qcol] = l_run; }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm_o[(size_t)wave * kOStride + (size_t)(dt * 16 + grp * 4 + i) * 16 + qcol] = o[dt][i];
  if constexpr (SHARE) {
    // the prompt's part of this row comes from the prefix workgroup (prompt s / G, this KV head): wait, bounded by the
    // wall clock, until its flag shows this launch's number; a wait that gives up sets the fault word, which makes the
    // sampler emit -1 for the step
    if (tid == 0) {
      const unsigned launch_no = (unsigned)(*rm.step) * (unsigned)sh.n_layers + (unsigned)sh.layer + 1u;
      const unsigned* flag = sh.flags + (size_t)(s / sh.G) * hkv + kvh;
      const unsigned long long t0 = wall_clock64();
      while ((int)(__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - launch_no) < 0) {
        if (wall_clock64() - t0 > sh.spin_ticks) {
          atomicOr(sh.fault, 2u);
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
  }
  __syncthreads();
  // thread -> (query head q, head dim d): one half of the X16 output (the query heads run fastest over the lanes: their
  // LDS columns are adjacent).  With one thread per 16-byte chunk only rep x HD / 8 threads - one wave - did the
  // whole merge, 80 dependent LDS reads each: 0.8 us at the end of a 4.5 us kernel.  Waves that had no page pair
  // carry (m = -inf, l = 0, o = 0) and drop out of the merge.
  const int KSo = (n_q_heads * HD) >> 5;
  for (int idx = tid; idx < rep * HD; idx += NW * 64) {
    const int q = idx % rep, d = idx / rep;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mx = fmaxf(mx, sm_m[w][q]);
    // the prefix part (shared-prompt variant): read past the L2, it was written by another workgroup of this launch
    float m_p = -INFINITY, l_p = 0.f, o_p = 0.f;
    if constexpr (SHARE) {
      const size_t base = ((size_t)s * n_q_heads + kvh * rep + q) * (HD + 4);
      m_p = ld_f32<true>(sh.pre, base * sizeof(float));
      l_p = ld_f32<true>(sh.pre, (base + 1) * sizeof(float));
      o_p = ld_f32<true>(sh.pre, (base + 4 + d) * sizeof(float));
      mx = fmaxf(mx, m_p);
    }
    const float w_p = SHARE ? __expf(m_p - mx) : 0.f;
    float den = w_p * l_p, wgt[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) { wgt[w] = __expf(sm_m[w][q] - mx); den += wgt[w] * sm_l[w][q]; }
    const float inv = 1.0f / den;
    float num = w_p * o_p;
#pragma unroll
    for (int w = 0; w < NW; ++w) num += wgt[w] * sm_o[(size_t)w * kOStride + (size_t)d * 16 + q];
    ((f16*)out)[x16_chunk(s, (kvh * rep + q) * HD + (d & ~7), KSo) * 8 + (d & 7)] = from_f32<f16>(num * inv);
  }
}

template <int HD, int NW, int PD, bool LDS = false, bool SHARE = false>
static hipError_t launch_decode_attention(const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* out, int S,
                                          int n_q_heads, hipStream_t st, const ShareArgs& sh = ShareArgs()) {
  static bool attr_done = false;
  static_assert(PD <= 4, "the LDS variant's waits cover up to 4 slots");
  const size_t smem = LDS ? (size_t)NW * PD * (HD / 8) * 1024
                          : (size_t)NW * HD * 16 * sizeof(float) + (SHARE ? (size_t)kSharePrefixMaxColumns * HD * sizeof(f16) : 0);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_decode_attention16<HD, NW, PD, LDS, SHARE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  return launch(SHARE ? KID_DECODE_ATTN_SHARED : KID_DECODE_ATTN, k_decode_attention16<HD, NW, PD, LDS, SHARE>,
                dim3((SHARE ? sh.n_prefix : 0) + S * kv.n_kv_heads), dim3(NW * 64), smem, st, qkv, rope, rm.step,
                kv.page_table, rm.Lp, kv.pages_per_seq, kv.n_kv_heads, n_q_heads, kv.k, rm, kv, (uint4*)out, sh);
}

hipError_t d_decode_attention(const float* qkv, const float2* rope, RowMap rm, KVCache kv, void* out, int S, int n_q_heads,
                              const ShareArgs* share, hipStream_t st) {
  if (share && share->prefix_pairs > 0) {
    // what the two-role launch assumes: rows are P x G sequences in order, all at one position, with their own
    // page-table rows; the columns of all siblings fit the prefix workgroup's four MFMA tiles
    const int rep = n_q_heads / kv.n_kv_heads;
    if (kv.head_dim != 64 || !rm.decode || rm.lens || rm.slot_seq || share->G < 1 || S % share->G != 0 ||
        share->G * rep > kSharePrefixMaxColumns || share->n_prefix != (S / share->G) * kv.n_kv_heads || !share->pre ||
        !share->flags || !share->fault || share->prefix_pairs * 32 > rm.Lp)
      return hipErrorInvalidValue;
    return launch_decode_attention<64, 8, 3, false, true>(qkv, rope, rm, kv, out, S, n_q_heads, st, *share);
  }
  // SAPO_ATTN_LDS=1 in the environment: the LDS-staged variant, kept as the measured alternative (0.5B-class decoder,
  // 64 sequences, same waves and pairs in flight: 6.6 against 5.8 us per launch at contexts 128..383, 12.5 against
  // 11.4 us at 512..1535).  Two slots of 8 KiB per wave are what 8 waves fit into the 160 KiB.  Read per call, so
  // that a test can switch it; a captured decode step keeps the variant it was captured with.
  const char* lds_env = getenv("SAPO_ATTN_LDS");
  if (kv.head_dim == 64) {
    if (lds_env && lds_env[0] == '1') return launch_decode_attention<64, 8, 2, true>(qkv, rope, rm, kv, out, S, n_q_heads, st);
    return launch_decode_attention<64, 8, 3>(qkv, rope, rm, kv, out, S, n_q_heads, st);
  }
  if (kv.head_dim == 128) {
    // more workgroups than compute units: 4-wave workgroups with one page pair in flight per wave leave room for
    // two per compute unit, so the whole grid is resident at once (1.5B, 256 sequences: 24.7 us against 29.8)
    if (S * kv.n_kv_heads > 256) return launch_decode_attention<128, 4, 1>(qkv, rope, rm, kv, out, S, n_q_heads, st);
    return launch_decode_attention<128, 8, 2>(qkv, rope, rm, kv, out, S, n_q_heads, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace sapo
