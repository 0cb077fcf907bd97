// Device functions of the decode step (gfx950) for the persistent per-step kernel of decode_persist.hip: the unit of
// work of a skinny GEMM and of the decode attention as functions a resident workgroup calls phase after phase (the
// kernels of kernels_decode.hip do the same work as one kernel per phase).  Operands are IEEE half in MFMA fragment order:
//   weights  W16[((tile * KS + ks) * 64 + lane)]           (uint4 = 8 half)
//            = W[tile*16 + lane%16][ks*32 + (lane/16)*8 .. +7],                       KS = K / 32
//   tokens   X16[(((tok/64) * KS + ks) * 4 + (tok/16)%4) * 64 + tok%16 + 16*((k%32)/8)]
//            = x[tok][ks*32 + ((k%32)/8)*8 .. +7]
// D = W-fragment x X-fragment leaves lane l with features (l/16)*4 .. +3 of token l%16.
//
// Every function takes a COH switch.  COH = false: one kernel per phase, plain loads and stores (a kernel boundary
// makes a producer's stores visible to its consumer).  COH = true: producer and consumer are workgroups of the SAME
// launch, possibly on different XCDs whose L2s do not see each other's lines inside a kernel: what another
// workgroup will read is stored write-through (sc0 sc1), what another workgroup wrote is loaded past the L2
// (sc0 sc1), and nothing is invalidated or written back wholesale (an L2 invalidate costs more than the step).
// These are buffer instructions with the cache-policy operand set (the compiler keeps its usual count of them).
#pragma once
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


struct NoWait { __device__ __forceinline__ void operator()() const {} };
// The thread's index as a value the compiler must take as new each time: inside a kernel that walks many phases in
// a loop, nothing derived from it (per-lane offsets of every phase) is then hoisted out of the loop and kept alive
// across all the other phases, which is what makes such a kernel spill.
__device__ __forceinline__ int fresh_thread_index() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

// ---------------------------------------------------------------------------------------
// Sum of the ssq parts of one token, spread over the 8 waves of a workgroup: thread (grp, tok)
// loads parts grp, grp + 8, ... (ssq_issue) and the sums meet in LDS later (ssq_publish, ssq_scale).
// ---------------------------------------------------------------------------------------
constexpr int kSsqPerThread = 12;   // up to 96 parts

template <bool COH>
__device__ __forceinline__ void ssq_issue(const float* __restrict__ ssq, int parts, int stride, int tok0,
                                          float (&sq)[kSsqPerThread]) {
  const int tok = threadIdx.x & 63, grp = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < kSsqPerThread; ++i) {
    const int p = grp + 8 * i;
    sq[i] = (ssq != nullptr && p < parts) ? ld_f32<COH>(ssq, ((size_t)p * stride + tok0 + tok) * sizeof(float)) : 0.f;
  }
}
// s_part: LDS [8][64].  Call before a __syncthreads(); ssq_scale() after it.
__device__ __forceinline__ void ssq_publish(const float (&sq)[kSsqPerThread], float* s_part) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kSsqPerThread; ++i) s += sq[i];
  s_part[threadIdx.x] = s;
}
__device__ __forceinline__ float ssq_scale(const float* s_part, int tok_local, int norm_dim, float eps) {
  float s = 0.f;
#pragma unroll
  for (int g = 0; g < 8; ++g) s += s_part[g * 64 + tok_local];
  return 1.0f / sqrtf(s / (float)norm_dim + eps);
}

// ---------------------------------------------------------------------------------------
// One unit of a skinny GEMM.  512 threads = 8 waves.
// The unit owns NT 16-feature tiles x TG 16-token groups (tokens tb * 64 + tg0 * 16 ...) over the whole K; wave w
// takes the k steps w, w + 8, ... (R of them per round, all loads of a round in flight at once), and the 8 partial
// results are summed through LDS in wave order, so a result depends neither on timing nor on the blocking
// (NT, TG, R only decide which workgroup computes a tile and how many loads are in flight).
// The first round's weight tiles are requested BEFORE wait_input() is called: weights do not depend on the
// activations, so in the persistent kernel they are on their way while the workgroup still waits for its input.
// Every wave calls wait_input() exactly once, whatever K is.
// LDS: red[8 waves][CH * TG][64 lanes] float4 with CH = (NT * TG > 16) ? 16 / TG : NT; s_part[512] floats.
// Epilogues:
//   STORE  : out_f32[tok][feat] = acc * scale(tok) (+ bias)
//   SWIGLU : tiles come in (gate, up) pairs; act = silu(gate * scale) * (up * scale) -> half, X16 order
//   RESID  : h[tok][feat] += acc;  xp_out = half(h * gain_next) in X16 order;  ssq_out[tile][tok] =
//            sum of h^2 over the tile's 16 features
// ---------------------------------------------------------------------------------------
constexpr int skinny_chunk_tiles(int NT, int TG) { return (NT * TG > 16) ? 16 / TG : NT; }
constexpr size_t skinny_red_bytes(int NT, int TG) { return (size_t)8 * skinny_chunk_tiles(NT, TG) * TG * 64 * sizeof(float4); }

template <int NT, int TG, int R, int MODE, bool COH, typename Wait>
__device__ __forceinline__ void skinny_unit(const SkinnyArgs& a, int unit, int tb, int tg0, float4* red, float* s_part,
                                            Wait wait_input) {
  constexpr int CH = skinny_chunk_tiles(NT, TG);
  static_assert(NT % CH == 0 && (MODE != SKM_SWIGLU || CH % 2 == 0), "tile chunking");
  constexpr int RS = (CH * TG * 64 + 511) / 512;   // output slots per thread and chunk
  const int tid = COH ? fresh_thread_index() : (int)threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int KS = a.K >> 5;
  const int tile0 = unit * NT;
  f32x4 acc[NT][TG];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int g = 0; g < TG; ++g) acc[t][g] = f32x4{0.f, 0.f, 0.f, 0.f};
  float sq[kSsqPerThread];
  if (!COH && MODE != SKM_RESID) ssq_issue<false>(a.ssq_in, a.ssq_parts, a.s_pad, tb * 64, sq);
  // RESID, single chunk: this thread's residual / gain operands are requested up front (the residual rows were
  // written at least one exchange ago)
  u32x4 h_old[RS];
  float4 g_next[RS];
  if (MODE == SKM_RESID && CH == NT) {
#pragma unroll
    for (int i = 0; i < RS; ++i) {
      const int slot = tid + 512 * i;
      h_old[i] = u32x4{0u, 0u, 0u, 0u};
      g_next[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (slot < NT * TG * 64) {
        const int t = slot / (TG * 64), g = (slot >> 6) % TG, l = slot & 63;
        const int tok = tb * 64 + (tg0 + g) * 16 + (l & 15);
        const int f0 = (tile0 + t) * 16 + (l >> 4) * 4;
        if (tok < a.n_rows) {
          h_old[i] = ld_u4<COH>(a.h, ((size_t)tok * a.N + f0) * sizeof(float));
          g_next[i] = *(const float4*)(a.gain_next + f0);
        }
      }
    }
  }

  const uint4* wbase = a.Wp + (size_t)tile0 * KS * 64 + lane;
  const size_t xoff = (((size_t)tb * KS * 4 + tg0) * 64 + lane) * sizeof(uint4);
  Frag16 wf[R][NT], xf[R][TG];
  auto load_w = [&](int k0) {
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int ks = k0 + 8 * i;
      if (ks < KS) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
          wf[i][t].n = __builtin_nontemporal_load((const u32x4*)(wbase + ((size_t)t * KS + ks) * 64));
      }
    }
  };
  load_w(wave);
  wait_input();
  if (COH && MODE != SKM_RESID) ssq_issue<true>(a.ssq_in, a.ssq_parts, a.s_pad, tb * 64, sq);
  for (int k0 = wave; k0 < KS; k0 += 8 * R) {
    if (k0 != wave) load_w(k0);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int ks = k0 + 8 * i;
      if (ks < KS) {
#pragma unroll
        for (int g = 0; g < TG; ++g) xf[i][g].n = ld_u4<COH>(a.Xp, xoff + (size_t)(ks * 4 + g) * 64 * sizeof(uint4));
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
  if (MODE != SKM_RESID) ssq_publish(sq, s_part);
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
        st_h4<COH>(a.xp_out, (x16_chunk(tok, f0, KSo) * 8 + (f0 & 4)) * sizeof(f16), o);
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
          st_f4<COH>(a.out_f32, ((size_t)tok * a.ldc + f0) * sizeof(float), o);
        }
      }
    } else {
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
          if (CH == NT) {
            ho = as_f4(h_old[i]); gn = g_next[i];
          } else {
            ho = as_f4(ld_u4<COH>(a.h, ((size_t)tok * a.N + f0) * sizeof(float)));
            gn = *(const float4*)(a.gain_next + f0);
          }
          s.x += ho.x; s.y += ho.y; s.z += ho.z; s.w += ho.w;
          st_f4<COH>(a.h, ((size_t)tok * a.N + f0) * sizeof(float), s);
          o[0] = from_f32<f16>(s.x * gn.x); o[1] = from_f32<f16>(s.y * gn.y);
          o[2] = from_f32<f16>(s.z * gn.z); o[3] = from_f32<f16>(s.w * gn.w);
          q = s.x * s.x + s.y * s.y + s.z * s.z + s.w * s.w;
        } else {
          o[0] = o[1] = o[2] = o[3] = (f16)0.f;
        }
        st_h4<COH>(a.xp_out, (x16_chunk(tok, f0, a.N >> 5) * 8 + (f0 & 4)) * sizeof(f16), o);
        q = sum_xor16(q);
        q = sum_xor32(q);
        if (l < 16) st_f32<COH>(a.ssq_out, ((size_t)(tile0 + c0 + t) * a.s_pad + tok) * sizeof(float), q);
      }
    }
  }
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
constexpr size_t attention_smem_bytes(int HD, int NW) {
  return (size_t)NW * HD * 16 * sizeof(float) + 2 * (size_t)NW * 16 * sizeof(float) + (size_t)(16 * HD + 2 * HD) * sizeof(f16);
}

// One (row s, KV head kvh) unit.  smem: attention_smem_bytes(HD, NW) bytes, 16-byte aligned.  K/V pages of the
// earlier tokens are requested before wait_input() is called (they were written by earlier launches); the row's
// q / k / v (qkv, possibly written by another workgroup of this launch) are read after it.
template <int HD, int NW, int PD, bool COH, typename Wait>
__device__ __forceinline__ void attention_unit(const float* __restrict__ qkv, const float2* __restrict__ rope, const RowMap& rm,
                                               const KVCache& kv, uint4* __restrict__ out, int n_q_heads, int s, int kvh,
                                               char* smem, Wait wait_input) {
  constexpr int KK = HD / 32;   // k steps of S^T = K Q^T
  constexpr int DT = HD / 16;   // 16-row tiles of O^T
  float* sm_o = (float*)smem;                                  // [NW][HD][16]
  float (*sm_m)[16] = (float (*)[16])(sm_o + (size_t)NW * HD * 16);
  float (*sm_l)[16] = sm_m + NW;
  f16* qs = (f16*)(sm_l + NW);                                 // [16][HD]
  f16* knew = qs + 16 * HD;
  f16* vnew = knew + HD;
  const int tid = COH ? fresh_thread_index() : (int)threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int qcol = lane & 15, grp = lane >> 4;
  const int hkv = kv.n_kv_heads, rep = n_q_heads / hkv;
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
  auto load_pair = [&](int pp, Frag16 (&kf)[2][KK], Frag16 (&vf)[DT]) {
    const int pa = pt[2 * pp];
    const int pb = pt[min(2 * pp + 1, last_page)];
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
  Frag16 kf[PD][2][KK], vf[PD][DT];
#pragma unroll
  for (int j = 0; j < PD; ++j)
    if (wave + NW * j < npairs) load_pair(wave + NW * j, kf[j], vf[j]);

  wait_input();
  // ---- rotary on the group's queries and the new key; append key / value -------------------
  {
    const int half = HD / 2;
    const int new_page = pt[pos / kPageTokens], new_slot = pos % kPageTokens;
    const size_t row = (size_t)s * (n_q_heads + 2 * hkv) * HD;   // float index of the row's first entry in qkv
    auto x_at = [&](size_t i) -> float { return ld_f32<COH>(qkv, (row + i) * sizeof(float)); };
    for (int idx = tid; idx < 16 * half; idx += NW * 64) {
      const int r = idx / half, i = idx % half;
      float r1 = 0.f, r2 = 0.f;
      if (r < rep) {
        const size_t x = (size_t)(kvh * rep + r) * HD;
        const float2 cs = rope[(size_t)pos * half + i];
        const float a = x_at(x + i), b = x_at(x + i + half);
        r1 = rot_first(a, b, cs.x, cs.y);
        r2 = rot_second(a, b, cs.x, cs.y);
      }
      qs[r * HD + i] = from_f32<f16>(r1);
      qs[r * HD + i + half] = from_f32<f16>(r2);
    }
    for (int i = tid; i < half; i += NW * 64) {
      const size_t x = (size_t)(n_q_heads + kvh) * HD;
      const float2 cs = rope[(size_t)pos * half + i];
      f16* kp = kpool + (size_t)new_page * page_elems + ((size_t)kvh * kPageTokens + new_slot) * HD;
      const float a = x_at(x + i), b = x_at(x + i + half);
      const f16 k1 = from_f32<f16>(rot_first(a, b, cs.x, cs.y)), k2 = from_f32<f16>(rot_second(a, b, cs.x, cs.y));
      kp[i] = k1; kp[i + half] = k2;
      knew[i] = k1; knew[i + half] = k2;
    }
    for (int i = tid; i < HD; i += NW * 64) {
      const f16 vv = from_f32<f16>(x_at((size_t)(n_q_heads + hkv + kvh) * HD + i));
      vpool[(size_t)new_page * page_elems + ((size_t)kvh * HD + i) * kPageTokens + new_slot] = vv;
      vnew[i] = vv;
    }
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

  for (int c0 = 0; wave + NW * c0 < npairs; c0 += PD) {
    if (c0 > 0) {
#pragma unroll
      for (int j = 0; j < PD; ++j)
        if (wave + NW * (c0 + j) < npairs) load_pair(wave + NW * (c0 + j), kf[j], vf[j]);
    }
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      const int pp = wave + NW * (c0 + j);
      if (pp >= npairs) break;
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
    for (int i = 0; i < 4; ++i) sm_o[((size_t)wave * HD + dt * 16 + grp * 4 + i) * 16 + qcol] = o[dt][i];
  __syncthreads();
  // thread -> (query q, 8 consecutive head dims): one 16-byte chunk of the X16 output.  Waves that
  // had no page pair carry (m = -inf, l = 0, o = 0) and drop out of the merge.
  const int KSo = (n_q_heads * HD) >> 5;
  for (int idx = tid; idx < rep * (HD / 8); idx += NW * 64) {
    const int q = idx / (HD / 8), d0 = (idx % (HD / 8)) * 8;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mx = fmaxf(mx, sm_m[w][q]);
    float den = 0.f, wgt[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) { wgt[w] = __expf(sm_m[w][q] - mx); den += wgt[w] * sm_l[w][q]; }
    const float inv = 1.0f / den;
    Frag16 ov;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float num = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) num += wgt[w] * sm_o[((size_t)w * HD + d0 + e) * 16 + q];
      ov.h[e] = from_f32<f16>(num * inv);
    }
    st_u4<COH>(out, x16_chunk(s, (kvh * rep + q) * HD + d0, KSo) * sizeof(uint4), ov.n);
  }
}


}  // namespace sapo
