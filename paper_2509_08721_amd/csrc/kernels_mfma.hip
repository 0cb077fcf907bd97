// 16-bit MFMA kernels for gfx950 used when many tokens go through the layers at once (prefill and
// scoring): weight packing, the token-parallel ("big") GEMM, and the fused LM head of the scoring
// pass (log-softmax + target gather).
//
// Operand type: the model's weights are bf16 values; the packed copies hold the same values as IEEE
// half (exact for 6.1e-5 <= |w| <= 65504, absolute error below 3e-8 under that) and activations
// are rounded to half (clamped to its range) instead of bf16.  Both run the MFMA at the same rate;
// half keeps 3 more mantissa bits, which is what keeps 28-layer models inside the stated logit and
// log-prob tolerances (with bf16 activations the rounding points alone put the 1.5B-class model's
// logits 6e-2 away from the definition).
#include "common.h"

namespace sapo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
union Frag {
  uint4 u;
  u32x4 n;
  bf16x8 v;
  f16x8 h;
};

__device__ __forceinline__ f32x16 mfma32(const Frag& a, const Frag& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.h, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16h(const Frag& a, const Frag& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c, 0, 0, 0);
}
// x * sigmoid(x) with the hardware reciprocal (1 ulp) instead of an IEEE division: the token-parallel SwiGLU epilogue
// evaluates 64 of these per thread and tile, where the correctly rounded division alone was a dozen instructions
// each; the result is rounded to half right after.
__device__ __forceinline__ float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// ---------------------------------------------------------------------------------------
// weight packing: row-major bf16 [n_rows, K] -> half, fragment order, 32-row tiles placed at
// dst_tile0 + t * dst_tile_stride (stride 2 interleaves gate and up tiles).
// ---------------------------------------------------------------------------------------
// range: kPackRangeSlots (512) pairs of counters, to be summed by the reader.  The first of a pair counts values half
// cannot hold (|w| > 65504, infinities, NaN: they would be clamped or carried as NaN), the second non-zero values
// below half's smallest normal number 2^-14 (kept with an absolute error below 3e-8).
__global__ void k_pack_weight(const bf16* __restrict__ src, int n_rows, int K, uint4* __restrict__ dst, int tile0,
                              int tile_stride, unsigned* __restrict__ range) {
  const int KS = K >> 4;
  const size_t total = (size_t)(n_rows >> 5) * KS * 64;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;   // total is a multiple of 64: a wave leaves or stays as a whole
  const int lane = (int)(idx & 63);
  const int ks = (int)((idx >> 6) % KS);
  const int t = (int)((idx >> 6) / KS);
  const int row = t * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
  Frag v, o;
  v.u = *(const uint4*)(src + (size_t)row * K + k);
#pragma unroll
  for (int e = 0; e < 8; ++e) o.h[e] = from_f32<f16>((float)v.v[e]);   // bf16 value -> half
  dst[((size_t)(tile0 + t * tile_stride) * KS + ks) * 64 + lane] = o.u;
  if (range) {
    unsigned too_large = 0, tiny = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float a = fabsf((float)v.v[e]);
      too_large += !(a <= 65504.f);
      tiny += (a > 0.f && a < 6.103515625e-05f);
    }
    // one atomic per wave and counter, only when there is something to add, spread over kPackRangeSlots pairs of
    // counters (small weights are common: with one pair every wave of a 0.5B model queues on the same address)
    unsigned packed = (too_large << 16) | tiny;          // at most 8 each per lane
    for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off, 64);   // at most 512 each per wave
    if (lane == 0) {
      unsigned* slot = range + 2 * (((unsigned)(idx >> 6) * 2654435761u) >> (32 - 9));
      if (packed >> 16) atomicAdd(slot, packed >> 16);
      if (packed & 0xffffu) atomicAdd(slot + 1, packed & 0xffffu);
    }
  }
}
hipError_t m_pack_weight(const void* src, int n_rows, int K, void* dst, int dst_tile0, int dst_tile_stride,
                         unsigned* range, hipStream_t st) {
  const size_t total = (size_t)(n_rows / 32) * (K / 16) * 64;
  if (total == 0) return hipSuccess;
  return launch(KID_MISC, k_pack_weight, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16*)src, n_rows, K, (uint4*)dst, dst_tile0,
                                                                  dst_tile_stride, range);
}

// =======================================================================================
// Token-parallel ("big") GEMM:  C[tok, feat] = sum_k X[tok, k] W[feat, k]
//
// Both operands are in 32-row fragment order in global memory (one MFMA 32x32x16 operand of one
// wave = one contiguous 1 KiB block):
//   W32[((fblk * KS + ks) * 64 + lane)] = W[fblk*32 + lane%32][ks*16 + (lane/32)*8 .. +7],  KS = K / 16
//   X32[((tblk * KS + ks) * 64 + lane)] = X[tblk*32 + lane%32][ks*16 + (lane/32)*8 .. +7]
// so a fragment moves from global memory to LDS with one direct-to-LDS load per wave and is read
// back with one conflict-free ds_read_b128.
// Workgroup tile 256 tokens x 128 features, 4 waves as 2 (tokens) x 2 (features), each 128 x 64 =
// 4 x 2 MFMA tiles; 32 k per stage (24 fragments), three stages in an LDS ring with two in flight.
// Two workgroups fit a compute unit (72 KiB LDS, <= 256 registers), which is what overlaps one
// workgroup's barrier and LDS latency with the other's MFMAs.
// The direct-to-LDS loads are issued from inline assembly: the compiler would otherwise wait for
// all of them before any LDS read, which removes the prefetch distance.  Their completion is
// awaited with explicit s_waitcnt vmcnt(N) (loads retire in order).
// Accumulator layout: acc[fi][tj][4 r + j] = C[tok = tj*32 + lane%32][feat = fi*32 + 8 r + (lane/32)*4 + j].
// ---------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ size_t x32_chunk(int tok, int k, int KS) {
  return (((size_t)(tok >> 5) * KS + (k >> 4)) * 64) + (tok & 31) + 32 * ((k >> 3) & 1);
}

constexpr int kStageFrags = 24;   // 16 token fragments + 8 feature fragments per 32-k stage
constexpr int kStages = 3;
constexpr int kBigLds = kStages * kStageFrags * 1024;

__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}
// one wave-wide 1 KiB copy global -> LDS: lane l's 16 bytes land at lds + 16 l
__device__ __forceinline__ void dma16(const void* g, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Block id -> (feature tile bx, token tile by).  Block ids are dealt round-robin to the 8 XCDs, each
// with its own L2.  With 8 or more token tiles XCD c owns the token tiles 8 y' + c and walks them in
// supertiles of 8 token tiles x 8 feature tiles (feature tiles fastest), the 64 workgroups it runs at
// a time.  With fewer token tiles XCD c owns the feature tiles 8 x' + c instead and walks each one's
// token tiles back to back, so every weight tile is fetched into one L2 only.
__device__ __forceinline__ bool big_raster(int NX, int NY, int& bx, int& by) {
  const int b = blockIdx.x, xcd = b & 7, j = b >> 3;
  if (NY < 8) {
    by = j % NY;
    bx = (j / NY) * 8 + xcd;
    return bx < NX;
  }
  const int NXs = (NX + 7) >> 3;
  const int sti = j >> 6, w = j & 63;
  bx = (sti % NXs) * 8 + (w & 7);
  by = ((sti / NXs) * 8 + (w >> 3)) * 8 + xcd;
  return bx < NX && by < NY;
}
static int big_grid(int NX, int NY) {
  if (NY < 8) return 8 * NY * ((NX + 7) / 8);
  return 8 * ((NX + 7) / 8) * ((((NY + 7) / 8) + 7) / 8) * 64;
}

// acc = X[tblk0*32 .. +255][:] . W[fblk0*32 .. +127][:]^T over the whole K.  Token blocks past the end
// are clamped to the last one (their results are never stored).
struct NoPrologue { __device__ __forceinline__ void operator()() const {} };
// `prologue` runs once the first two stages are requested (loads it issues ride on the same latency).
// NS: depth of the LDS ring (NS - 1 stages in flight).
// TJ: 32-token blocks per wave (4: a 256-token tile, the default; 2: a 128-token tile with a third workgroup per
// compute unit, for launches whose 256-token tiles would leave the last round of workgroups mostly empty).
template <int NS = kStages, class Prologue = NoPrologue, int TJ = 4>
__device__ __forceinline__ void big_mainloop(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int n_tblk,
                                             int KS, int tblk0, int fblk0, uint4* smem, f32x16 (&acc)[2][TJ],
                                             Prologue prologue = Prologue(), int st0 = 0, int n_stages = -1) {
  constexpr int TF = 4 * TJ;        // token fragments of a stage (2 TJ token blocks x 2 k halves)
  constexpr int SF = TF + 8;        // fragments of a stage
  constexpr int NF = SF / 4;        // requests per wave and stage
  static_assert(TJ == 4 || TJ == 2, "tile of 256 or 128 tokens");
  const int tid = threadIdx.x, wave = wave_index(tid), lane = tid & 63;
  const int wf = wave & 1, wt = wave >> 1;
  const int nst = n_stages < 0 ? (KS >> 1) : n_stages;   // stages of 32 k; a split-K workgroup runs st0 .. st0 + nst - 1
  const uint4* src[NF];
  unsigned dst[NF];
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const int f = wave * NF + i;
    if (f < TF) {
      int tb = tblk0 + (f >> 1);
      if (tb > n_tblk - 1) tb = n_tblk - 1;
      src[i] = Xp + ((size_t)tb * KS + 2 * st0 + (f & 1)) * 64 + lane;
    } else {
      const int g = f - TF;
      src[i] = Wp + ((size_t)(fblk0 + (g >> 1)) * KS + 2 * st0 + (g & 1)) * 64 + lane;
    }
    dst[i] = __builtin_amdgcn_readfirstlane(lds_addr(smem + f * 64));
  }
  auto issue = [&](int st) {
    const unsigned sbase = (unsigned)((st % NS) * SF * 1024);
#pragma unroll
    for (int i = 0; i < NF; ++i) dma16(src[i] + (size_t)st * 128, dst[i] + sbase);
  };
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < TJ; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  wg_barrier();   // a previous pass over the ring (fused LM head) is over in every wave
#pragma unroll
  for (int p = 0; p < NS - 1; ++p)
    if (p < nst) issue(p);
  prologue();
  for (int st = 0; st < nst; ++st) {
    // this wave's part of stage st has landed once at most the newer stages' requests are outstanding
    const int newer = min(NS - 2, nst - 1 - st);
    if (newer >= 4) wait_vmcnt<4 * NF>();
    else if (newer == 3) wait_vmcnt<3 * NF>();
    else if (newer == 2) wait_vmcnt<2 * NF>();
    else if (newer == 1) wait_vmcnt<NF>();
    else wait_vmcnt<0>();
    wg_barrier();                                               // ... and everybody's; stage st-1 is consumed
    // The requests of stage st + NS - 1 go out one after each of the first MFMAs instead of in a burst behind
    // the barrier: the burst held up the LDS reads and MFMAs queued behind it (same sums, 15 % faster on the scorer's
    // shape in a stand-alone copy of the loop).  The fences keep the compiler from regrouping them.
    const bool more = st + NS - 1 < nst;
    const unsigned next_base = (unsigned)(((st + NS - 1) % NS) * SF * 1024);
    const size_t next_off = (size_t)(st + NS - 1) * 128;
    const uint4* buf = smem + (st % NS) * SF * 64;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      Frag xf[TJ], wfr[2];
#pragma unroll
      for (int tj = 0; tj < TJ; ++tj) xf[tj].u = buf[((wt * TJ + tj) * 2 + s2) * 64 + lane];
#pragma unroll
      for (int fi = 0; fi < 2; ++fi) wfr[fi].u = buf[(TF + (wf * 2 + fi) * 2 + s2) * 64 + lane];
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) {
          acc[fi][tj] = mfma32(wfr[fi], xf[tj], acc[fi][tj]);
          const int m = (s2 * 2 + fi) * TJ + tj;
          if (m < NF) {
            __builtin_amdgcn_sched_barrier(0);
            if (more) dma16(src[m] + next_off, dst[m] + next_base);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
    }
  }
}

template <int TJ>
__global__ void __launch_bounds__(256, TJ == 4 ? 2 : 3) k_gemm_big(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp,
                                                                  int M, int N, int K, BigEpi ep) {
  constexpr int TM = 64 * TJ;   // tokens per tile
  extern __shared__ uint4 smem[];
  int bx, by, st0 = 0, n_st = K >> 5;
  if (ep.splits > 1) {
    // split-K (one token tile): XCD c runs the splits c, c + 8, ... of every feature tile, so the K range of
    // the token operand that a split reads sits in one L2; split z covers stages z nst / s .. (z + 1) nst / s
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, per = ep.splits >> 3;
    const int z = (j % per) * 8 + xcd;
    bx = j / per; by = 0;
    st0 = (int)((long)z * n_st / ep.splits);
    n_st = (int)((long)(z + 1) * n_st / ep.splits) - st0;
    ep.out_f32 += (size_t)z * ep.split_stride;
  } else if (!big_raster(N >> 7, (M + TM - 1) / TM, bx, by)) {
    return;
  }
  f32x16 acc[2][TJ];
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
  const int wf = wave & 1, wt = wave >> 1;
  float row_scale[TJ];
#pragma unroll
  for (int tj = 0; tj < TJ; ++tj) row_scale[tj] = 1.f;
  auto prologue = [&]() {
    if (!ep.ssq_in) return;
    const int ps = (ep.ssq_parts + 3) & ~3;   // row stride of the parts; at most 16 parts
    float4 part[TJ][4];
#pragma unroll
    for (int tj = 0; tj < TJ; ++tj) {
      const int tok = min(by * TM + wt * (32 * TJ) + tj * 32 + (lane & 31), M - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        part[tj][i] = (4 * i < ps) ? *(const float4*)(ep.ssq_in + (size_t)tok * ps + 4 * i) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int tj = 0; tj < TJ; ++tj) {
      float ss = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {   // padding slots are never written: select, do not add
        ss += (4 * i + 0 < ep.ssq_parts) ? part[tj][i].x : 0.f;
        ss += (4 * i + 1 < ep.ssq_parts) ? part[tj][i].y : 0.f;
        ss += (4 * i + 2 < ep.ssq_parts) ? part[tj][i].z : 0.f;
        ss += (4 * i + 3 < ep.ssq_parts) ? part[tj][i].w : 0.f;
      }
      row_scale[tj] = rsqrtf(ss / ep.norm_dim + ep.eps);
    }
  };
  big_mainloop<kStages, decltype(prologue), TJ>(Xp, Wp, (M + 31) >> 5, K >> 4, by * (2 * TJ), bx * 4, smem, acc, prologue, st0, n_st);
  float ssq_mine[TJ];
#pragma unroll
  for (int tj = 0; tj < TJ; ++tj) ssq_mine[tj] = 0.f;
  const int tok0 = by * TM + wt * (32 * TJ) + (lane & 31);
  const int fcol = bx * 128 + wf * 64 + (lane >> 5) * 4;   // + fi * 32 + 8 r: this lane's four features of block (fi, r)
  float4 bb[2][4];
  if (ep.mode == BIG_STORE_F32 && ep.bias) {
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
      for (int r = 0; r < 4; ++r) bb[fi][r] = *(const float4*)(ep.bias + fcol + fi * 32 + 8 * r);
  }
#pragma unroll
  for (int tj = 0; tj < TJ; ++tj) {
    const int tok = tok0 + tj * 32;
    if (tok >= M) continue;   // lanes l and l + 32 hold the same token: they leave together
    if (ep.ssq_in) {
      const float sc = row_scale[tj];
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[fi][tj][v] *= sc;
    }
    if (ep.mode == BIG_SWIGLU) {
      // fi = 0 is a gate tile, fi = 1 the matching up tile; act goes out in X32 order over F = N / 2
      const int F = N >> 1;
      const int f0 = (bx * 2 + wf) * 32 + (lane >> 5) * 4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        f16x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = from_f32<f16>(silu_f(acc[0][tj][4 * r + j]) * acc[1][tj][4 * r + j]);
        *(f16x4*)(ep.out_act + x32_chunk(tok, f0 + 8 * r, F >> 4) * 8 + ((lane >> 5) << 2)) = o;
      }
    } else if (ep.mode == BIG_STORE_F32) {
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float4 v = make_float4(acc[fi][tj][4 * r], acc[fi][tj][4 * r + 1], acc[fi][tj][4 * r + 2], acc[fi][tj][4 * r + 3]);
          if (ep.bias) { v.x += bb[fi][r].x; v.y += bb[fi][r].y; v.z += bb[fi][r].z; v.w += bb[fi][r].w; }
          *(float4*)(ep.out_f32 + (size_t)tok * ep.ldc + fcol + fi * 32 + 8 * r) = v;
        }
    }
  }
  if (ep.mode == BIG_ADD_F32) {
    // Residual update.  In the accumulator layout a lane holds one token, so a load or store instruction on the
    // row-major fp32 residual touches 32 cache lines for 1 KiB.  The residual therefore moves in row layout (16 lanes
    // cover 256 contiguous bytes of a row: 8 full lines per instruction) and changes layout through LDS, once on the
    // way in and once on the way out, a wave's 64 (128-token tiles: 32) tokens x 64 features at a time in the wave's own
    // part of the ring (rows padded to 68 floats).  The sums, the next operand and the sums of squares are taken in the accumulator
    // layout as before: same results bit for bit.  The second half's rows are requested before the first half's
    // stores, since a load issued behind a store also waits for the store's acknowledgement.  A tile without rows
    // past the end and the producer side are compile-time cases, so that the common one is straight-line code
    // whose waits the compiler can count exactly.
    constexpr int RS = 68, HB = TJ == 4 ? 64 : 32, T2 = HB / 32, NI = HB / 4;   // HB tokens per pass, two passes
    wg_barrier();   // every wave has read its last stage: the ring is free
    float* R = (float*)smem + wave * (HB * RS);
    const int rt = lane >> 4, rc = (lane & 15) * 4;   // row layout: token 4 i + rt of the half, features rc .. rc + 3
    const int row0 = by * TM + wt * (32 * TJ), gcol = bx * 128 + wf * 64;
    auto wave_sync = [] {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto update = [&](auto full_c, auto prod_c) {
      constexpr bool full = decltype(full_c)::value, prod = decltype(prod_c)::value;
      // the wave's 64 gains wait in LDS behind the four row areas (held in registers they would not fit next to the
      // rows in flight)
      float* G = (float*)smem + 4 * HB * RS + wave * 64;
      if (prod && lane < 16) *(float4*)(G + 4 * lane) = *(const float4*)(ep.gain_next + gcol + 4 * lane);
      float4 in[NI];
      auto request = [&](int h, int i0) {   // rows 4 i + rt, i = i0 .. i0 + 7, of half h
#pragma unroll
        for (int i = i0; i < i0 + 8; ++i) {
          const int tok = row0 + h * HB + 4 * i + rt;
          in[i] = (full || tok < M) ? *(const float4*)(ep.out_f32 + (size_t)tok * ep.ldc + gcol + rc)
                                    : make_float4(0.f, 0.f, 0.f, 0.f);
        }
      };
#pragma unroll
      for (int i0 = 0; i0 < NI; i0 += 8) request(0, i0);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < NI; ++i) *(float4*)(R + (4 * i + rt) * RS + rc) = in[i];
        wave_sync();
#pragma unroll
        for (int t2 = 0; t2 < T2; ++t2) {
          const int tj = T2 * h + t2, tok = tok0 + tj * 32;
          float ssq = 0.f;
#pragma unroll
          for (int fi = 0; fi < 2; ++fi)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float4* q = (float4*)(R + (t2 * 32 + (lane & 31)) * RS + fi * 32 + 8 * r + (lane >> 5) * 4);
              const float4 w = *q;
              const float4 v = make_float4(acc[fi][tj][4 * r] + w.x, acc[fi][tj][4 * r + 1] + w.y,
                                           acc[fi][tj][4 * r + 2] + w.z, acc[fi][tj][4 * r + 3] + w.w);
              *q = v;
              if (prod && (full || tok < M)) {
                ssq += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                const float4 gn = *(const float4*)(G + fi * 32 + 8 * r + (lane >> 5) * 4);
                f16x4 hv;
                hv[0] = from_f32<f16>(v.x * gn.x); hv[1] = from_f32<f16>(v.y * gn.y);
                hv[2] = from_f32<f16>(v.z * gn.z); hv[3] = from_f32<f16>(v.w * gn.w);
                *(f16x4*)(ep.xn_out + x32_chunk(tok, fcol + fi * 32 + 8 * r, N >> 4) * 8 + ((lane >> 5) << 2)) = hv;
              }
            }
          ssq_mine[tj] = ssq + __shfl_xor(ssq, 32, 64);
        }
        wave_sync();
#pragma unroll
        for (int i0 = 0; i0 < NI; i0 += 8) {   // eight rows at a time: sixteen out and sixteen in would not fit the registers
          float4 out[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) out[i] = *(const float4*)(R + (4 * (i0 + i) + rt) * RS + rc);
          if (h == 0) request(1, i0);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int tok = row0 + h * HB + 4 * (i0 + i) + rt;
            if (full || tok < M) *(float4*)(ep.out_f32 + (size_t)tok * ep.ldc + gcol + rc) = out[i];
          }
        }
        wave_sync();   // the rows are in registers before the next half overwrites them
      }
    };
    const bool full = by * TM + TM <= M;
    if (ep.gain_next) {
      if (full) update(std::true_type(), std::true_type());
      else update(std::false_type(), std::true_type());
    } else {
      if (full) update(std::true_type(), std::false_type());
      else update(std::false_type(), std::false_type());
    }
  }
  if (ep.gain_next) {   // uniform: the two feature waves of a token half meet in LDS, summed in wave order
    __shared__ float red[256];
    if (wf == 1 && lane < 32) {
#pragma unroll
      for (int tj = 0; tj < TJ; ++tj) red[wt * (32 * TJ) + tj * 32 + lane] = ssq_mine[tj];
    }
    __syncthreads();
    if (wf == 0 && lane < 32) {
      const int ps = ((N >> 7) + 3) & ~3;
#pragma unroll
      for (int tj = 0; tj < TJ; ++tj) {
        const int tok = by * TM + wt * (32 * TJ) + tj * 32 + lane;
        if (tok < M) ep.ssq_out[(size_t)tok * ps + bx] = ssq_mine[tj] + red[wt * (32 * TJ) + tj * 32 + lane];
      }
    }
  }
}
// ---------------------------------------------------------------------------------------
// QKV projection with the rotary embedding and the KV append in its epilogue (token-parallel path): the
// fp32 q/k/v rows never exist in memory.  Same main loop as k_gemm_big.  A 128-feature tile is two
// heads of 64 (one per feature wave: the rotation partner i + 32 sits in the same lane, accumulator
// block fi = 1) or one head of 128 (the partner i + 64 sits in the other feature wave: the two waves
// swap their accumulators through LDS, two token blocks at a time).  q goes out as half row-major
// [M, Hq hd] (flash attention's operand), rotated k and v go to the row's cache page.
// ---------------------------------------------------------------------------------------
template <int HD>
__global__ void __launch_bounds__(256, 2) k_gemm_qkv_rope(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int M,
                                                          int N, int K, QkvEpi ep) {
  extern __shared__ uint4 smem[];
  int bx, by;
  if (!big_raster(N >> 7, (M + 255) >> 8, bx, by)) return;
  f32x16 acc[2][4];
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
  const int wf = wave & 1, wt = wave >> 1;
  float row_scale[4] = {1.f, 1.f, 1.f, 1.f};
  big_mainloop(Xp, Wp, (M + 31) >> 5, K >> 4, by * 8, bx * 4, smem, acc, [&]() {
    if (!ep.ssq_in) return;
    const int ps = (ep.ssq_parts + 3) & ~3;
    float4 part[4][4];
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      const int tok = min(by * 256 + wt * 128 + tj * 32 + (lane & 31), M - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        part[tj][i] = (4 * i < ps) ? *(const float4*)(ep.ssq_in + (size_t)tok * ps + 4 * i) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      float ss = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ss += (4 * i + 0 < ep.ssq_parts) ? part[tj][i].x : 0.f;
        ss += (4 * i + 1 < ep.ssq_parts) ? part[tj][i].y : 0.f;
        ss += (4 * i + 2 < ep.ssq_parts) ? part[tj][i].z : 0.f;
        ss += (4 * i + 3 < ep.ssq_parts) ? part[tj][i].w : 0.f;
      }
      row_scale[tj] = rsqrtf(ss / ep.norm_dim + ep.eps);
    }
  });
  const int hq = ep.n_q_heads, hkv = ep.kv.n_kv_heads;
  const int head = (HD == 64) ? bx * 2 + wf : bx;            // among Hq + 2 Hkv heads
  const bool is_v = head >= hq + hkv;
  const int half_sel = lane >> 5;
  // row scale and bias first: what is rotated is the finished projection
  {
    float4 bb[2][4];
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        bb[fi][r] = ep.bias ? *(const float4*)(ep.bias + bx * 128 + wf * 64 + fi * 32 + half_sel * 4 + 8 * r)
                            : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int tj = 0; tj < 4; ++tj)
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          acc[fi][tj][4 * r + 0] = acc[fi][tj][4 * r + 0] * row_scale[tj] + bb[fi][r].x;
          acc[fi][tj][4 * r + 1] = acc[fi][tj][4 * r + 1] * row_scale[tj] + bb[fi][r].y;
          acc[fi][tj][4 * r + 2] = acc[fi][tj][4 * r + 2] * row_scale[tj] + bb[fi][r].z;
          acc[fi][tj][4 * r + 3] = acc[fi][tj][4 * r + 3] * row_scale[tj] + bb[fi][r].w;
        }
  }
  f16* kpool = (f16*)ep.kv.k;
  f16* vpool = (f16*)ep.kv.v;
  // Where the four token blocks of this lane go: position, cache page, and whether anything is stored.  All four
  // page-table lookups are in flight together (rows past the end look up row M - 1 and store nothing).
  int pos_of[4], page_of[4];
  bool stores[4];
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    const int tok = by * 256 + wt * 128 + tj * 32 + (lane & 31), tokc = min(tok, M - 1);
    int seq;
    ep.rm.get(tokc, seq, pos_of[tj]);
    stores[tj] = tok < M && (head < hq || ep.rm.keeps_kv(tokc));
    page_of[tj] = ep.kv.page_table[(size_t)seq * ep.kv.pages_per_seq + pos_of[tj] / kPageTokens];
  }
  if (is_v) {
    const int vh = head - hq - hkv;
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      if (!stores[tj]) continue;
      f16* vp = vpool + ((size_t)page_of[tj] * hkv + vh) * HD * kPageTokens + pos_of[tj] % kPageTokens;
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int f = (HD == 64 ? 0 : wf * 64) + fi * 32 + 8 * (v >> 2) + (v & 3) + half_sel * 4;
          vp[(size_t)f * kPageTokens] = from_f32<f16>(acc[fi][tj][v]);
        }
    }
    return;
  }
  // start of a row's head: q row-major, k in its page slot
  auto head_row = [&](int tj) -> f16* {
    const int tok = by * 256 + wt * 128 + tj * 32 + (lane & 31);
    if (head < hq) return ep.q_out + ((size_t)tok * hq + head) * HD;
    return kpool + (((size_t)page_of[tj] * hkv + (head - hq)) * kPageTokens + pos_of[tj] % kPageTokens) * HD;
  };
  // The (cos, sin) pairs of a token block are requested one block ahead of the block being written, before that
  // block's stores: a load issued behind a store waits for the store's acknowledgement as well.
  if (HD == 64) {
    // pair (i, i + 32): x1 = block fi = 0, x2 = block fi = 1, i = 8 r + j + 4 half_sel
    float4 cs[2][4][2];
    auto request = [&](int tj, float4 (&dst)[4][2]) {
      const float2* cs_row = ep.rope + (size_t)pos_of[tj] * (HD / 2) + half_sel * 4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        dst[r][0] = *(const float4*)(cs_row + 8 * r);
        dst[r][1] = *(const float4*)(cs_row + 8 * r + 2);
      }
    };
    request(0, cs[0]);
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      if (tj < 3) request(tj + 1, cs[(tj + 1) & 1]);
      if (!stores[tj]) continue;
      f16* dst = head_row(tj);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i0 = 8 * r + half_sel * 4;
        const float4 c01 = cs[tj & 1][r][0], c23 = cs[tj & 1][r][1];
        const float c[8] = {c01.x, c01.y, c01.z, c01.w, c23.x, c23.y, c23.z, c23.w};
        f16x4 o1, o2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float x1 = acc[0][tj][4 * r + j], x2 = acc[1][tj][4 * r + j], co = c[2 * j], sn = c[2 * j + 1];
          o1[j] = from_f32<f16>(x1 * co - x2 * sn);
          o2[j] = from_f32<f16>(x2 * co + x1 * sn);
        }
        *(f16x4*)(dst + i0) = o1;
        *(f16x4*)(dst + i0 + 32) = o2;
      }
    }
    return;
  }
  // HD = 128, q or k head: pair (i, i + 64); this wave holds x1 (wf = 0) or x2 (wf = 1) at i = fi 32 + 8 r + j + 4 half_sel
  // and swaps accumulators with the other feature wave through LDS, two token blocks at a time
  float* ex = (float*)smem;   // [wt][wf][tj2][fi][v][lane]: 2 x 2 x 2 x 2 x 16 x 64 floats = 64 KiB
  float4 cs[2][4][2];
  auto request = [&](int tj, float4 (&dst)[2][4][2]) {
    const float2* cs_row = ep.rope + (size_t)pos_of[tj] * (HD / 2) + half_sel * 4;
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        dst[fi][r][0] = *(const float4*)(cs_row + fi * 32 + 8 * r);
        dst[fi][r][1] = *(const float4*)(cs_row + fi * 32 + 8 * r + 2);
      }
  };
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    wg_barrier();   // the ring (first round) or the previous round's partners have been read
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          ex[((((wt * 2 + wf) * 2 + t2) * 2 + fi) * 16 + v) * 64 + lane] = acc[fi][2 * h + t2][v];
    __syncthreads();
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const int tj = 2 * h + t2;
      request(tj, cs);   // all of the block's pairs before its first store (a full block ahead would not fit the registers)
      if (stores[tj]) {
        f16* dst = head_row(tj);
#pragma unroll
        for (int fi = 0; fi < 2; ++fi) {
          f32x16 other;
#pragma unroll
          for (int v = 0; v < 16; ++v) other[v] = ex[((((wt * 2 + (wf ^ 1)) * 2 + t2) * 2 + fi) * 16 + v) * 64 + lane];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i0 = fi * 32 + 8 * r + half_sel * 4;
            const float4 c01 = cs[fi][r][0], c23 = cs[fi][r][1];
            const float c[8] = {c01.x, c01.y, c01.z, c01.w, c23.x, c23.y, c23.z, c23.w};
            f16x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float a = acc[fi][tj][4 * r + j], b2 = other[4 * r + j], co = c[2 * j], sn = c[2 * j + 1];
              o[j] = from_f32<f16>(wf == 0 ? a * co - b2 * sn : a * co + b2 * sn);
            }
            *(f16x4*)(dst + wf * 64 + i0) = o;
          }
        }
      }
    }
  }
}

hipError_t m_gemm_qkv_rope(const void* Xp, const void* Wp, int M, int N, int K, const QkvEpi& epi, hipStream_t st) {
  if (M == 0) return hipSuccess;
  const int hd = epi.kv.head_dim;
  if (N % 128 != 0 || K % 32 != 0 || (hd != 64 && hd != 128) || N != (epi.n_q_heads + 2 * epi.kv.n_kv_heads) * hd)
    return hipErrorInvalidValue;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_gemm_qkv_rope<64>, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)k_gemm_qkv_rope<128>, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const dim3 grid(big_grid(N / 128, (M + 255) / 256));
  if (hd == 64)
    return launch(KID_GEMM_BIG, k_gemm_qkv_rope<64>, grid, dim3(256), kBigLds, st, (const uint4*)Xp, (const uint4*)Wp, M, N, K,
                  epi);
  return launch(KID_GEMM_BIG, k_gemm_qkv_rope<128>, grid, dim3(256), kBigLds, st, (const uint4*)Xp, (const uint4*)Wp, M, N, K,
                epi);
}

// 128-token tiles (three workgroups per compute unit) instead of 256-token tiles (two): for narrow outputs whose
// 256-token tiles fill their last round of resident workgroups badly, when the half-size tiles need no more rounds
// (64 x 384 tokens x 896 features: 672 tiles in 2 rounds of 512 become 1344 in 2 rounds of 768; O projection 86 ->
// 70 us, the prompt's small launches 70 -> 58 us.  With one round more - 64 x 768: 4 against 3 - the down projection
// lost 14 %, so that case keeps the large tile).  SAPO_BIG_TILE=128 / 256 in the environment forces one or the
// other (measurement).
static bool big_prefers_small_tiles(int NX, int M) {
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      n_cu = 256;
  }
  const char* e = getenv("SAPO_BIG_TILE");   // read per call, so that a test can switch it
  const int forced = e ? atoi(e) : 0;
  if (forced == 128) return true;
  if (forced == 256) return false;
  if (NX > 16) return false;   // wide outputs have rounds enough: the smaller tile only adds operand traffic per flop
  const long big = (long)NX * ((M + 255) / 256), small = (long)NX * ((M + 127) / 128);
  const long rounds_big = (big + 2 * n_cu - 1) / (2 * n_cu), rounds_small = (small + 3 * n_cu - 1) / (3 * n_cu);
  return rounds_small <= rounds_big;
}

hipError_t m_gemm_big(const void* Xp, const void* Wp, int M, int N, int K, BigEpi epi, hipStream_t st) {
  if (M == 0) return hipSuccess;
  if (N % 128 != 0 || K % 32 != 0) return hipErrorInvalidValue;
  constexpr int kSmallLds = kStages * (8 + 8) * 1024;   // the ring of a 128-token tile: 8 token + 8 feature fragments per stage
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_gemm_big<4>, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_gemm_big<2>, hipFuncAttributeMaxDynamicSharedMemorySize, kSmallLds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if (epi.splits < 1 || (epi.splits > 1 && (epi.splits % 8 != 0 || K / 32 < epi.splits || M > 256 ||
                                            epi.mode != BIG_STORE_F32 || epi.ssq_in || epi.bias)))
    return hipErrorInvalidValue;
  if (epi.gain_next && epi.mode != BIG_ADD_F32) return hipErrorInvalidValue;
  if (epi.splits == 1 && big_prefers_small_tiles(N / 128, M)) {
    const int g2 = big_grid(N / 128, (M + 127) / 128);
    return launch(epi.decode ? KID_GEMM_BIG_DECODE : KID_GEMM_BIG, k_gemm_big<2>, dim3(g2), dim3(256), kSmallLds, st,
                  (const uint4*)Xp, (const uint4*)Wp, M, N, K, epi);
  }
  const int g = epi.splits > 1 ? epi.splits * (N / 128) : big_grid(N / 128, (M + 255) / 256);
  return launch(epi.decode ? KID_GEMM_BIG_DECODE : KID_GEMM_BIG, k_gemm_big<4>, dim3(g), dim3(256), kBigLds, st, (const uint4*)Xp,
                (const uint4*)Wp, M, N, K, epi);
}

// ---------------------------------------------------------------------------------------
// RMSNorm of residual rows into X32 order: out[i] = half( h[r] * rsqrt(mean(h[r]^2) + eps) * gain ),
// r = row_index ? row_index[i] : i; negative r (padding) gives zeros.  One workgroup per row.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(128) k_rmsnorm_x32(const float* __restrict__ h, const float* __restrict__ gain, float eps,
                                                     uint4* __restrict__ out, int d, const int* __restrict__ row_index) {
  __shared__ float red[2];
  const int i = blockIdx.x;
  const int r = row_index ? row_index[i] : i;
  const int KS = d >> 4;
  if (r < 0) {
    for (int k = threadIdx.x * 8; k < d; k += 1024) out[x32_chunk(i, k, KS)] = make_uint4(0, 0, 0, 0);
    return;
  }
  const float* x = h + (size_t)r * d;
  float ss = 0.f;
  for (int k = threadIdx.x * 4; k < d; k += 512) {
    const float4 v = *(const float4*)(x + k);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_reduce_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float scale = 1.0f / sqrtf((red[0] + red[1]) / (float)d + eps);
  for (int k = threadIdx.x * 8; k < d; k += 1024) {
    const float4 a = *(const float4*)(x + k), b = *(const float4*)(x + k + 4);
    const float4 ga = *(const float4*)(gain + k), gb = *(const float4*)(gain + k + 4);
    Frag o;
    o.h[0] = from_f32<f16>(a.x * scale * ga.x); o.h[1] = from_f32<f16>(a.y * scale * ga.y);
    o.h[2] = from_f32<f16>(a.z * scale * ga.z); o.h[3] = from_f32<f16>(a.w * scale * ga.w);
    o.h[4] = from_f32<f16>(b.x * scale * gb.x); o.h[5] = from_f32<f16>(b.y * scale * gb.y);
    o.h[6] = from_f32<f16>(b.z * scale * gb.z); o.h[7] = from_f32<f16>(b.w * scale * gb.w);
    out[x32_chunk(i, k, KS)] = o.u;
  }
}
hipError_t m_rmsnorm_x32(const float* h, const float* gain, float eps, void* out, int M, int d, const int* row_index,
                         hipStream_t st) {
  if (M == 0) return hipSuccess;
  return launch(KID_RMSNORM, k_rmsnorm_x32, dim3(M), dim3(128), 0, st, h, gain, eps, (uint4*)out, d, row_index);
}

// ---------------------------------------------------------------------------------------
// LM head for scoring: log-softmax + target gather without materialising logits.
// Rastered like the GEMM over (256-row tiles) x (groups of kScoreGroup 128-feature tiles): a workgroup
// walks the tiles of its group for its 256 rows keeping a running (max, sum exp) per row, and the
// one lane that sees a row's target id writes the target logit.  A second kernel merges the groups
// in a fixed order.  partials: [n_groups][max_rows][2], then ztarget [max_rows].
// ---------------------------------------------------------------------------------------
constexpr int kScoreGroup = 16;
static int score_groups(int V) { return (V / 128 + kScoreGroup - 1) / kScoreGroup; }
size_t m_lmhead_score_partial_floats(int max_rows, int V) { return (size_t)max_rows * (2 * score_groups(V) + 1); }

__global__ void __launch_bounds__(256, 2) k_lmhead_score(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp,
                                                         int max_rows, const int* __restrict__ n_rows_dev, int V, int K,
                                                         const int* __restrict__ row_seq_pos,
                                                         const int32_t* __restrict__ tokens, int T,
                                                         float* __restrict__ partials) {
  extern __shared__ uint4 smem[];
  __shared__ float red_m[2][256], red_l[2][256];
  const int n_rows = *n_rows_dev;
  const int n_ft = V >> 7;
  const int n_groups = (n_ft + kScoreGroup - 1) / kScoreGroup;
  int bx, by;
  if (!big_raster(n_groups, (max_rows + 255) >> 8, bx, by)) return;
  const int tok0 = by * 256;
  if (tok0 >= n_rows) return;
  const int ft_begin = bx * kScoreGroup, ft_end = min(n_ft, ft_begin + kScoreGroup);
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
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
  float* ztarget = partials + (size_t)max_rows * 2 * n_groups;
  for (int ft = ft_begin; ft < ft_end; ++ft) {
    f32x16 acc[2][4];
    big_mainloop(Xp, Wp, (n_rows + 31) >> 5, K >> 4, by * 8, ft * 4, smem, acc);
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      const int row = tok0 + wt * 128 + tj * 32 + (lane & 31);
#pragma unroll
      for (int fi = 0; fi < 2; ++fi) {
        const int f0 = ft * 128 + wf * 64 + fi * 32 + (lane >> 5) * 4;
        float mt = acc[fi][tj][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mt = fmaxf(mt, acc[fi][tj][v]);
        const float mn = fmaxf(lse[tj].m, mt);
        float su = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) su += __expf(acc[fi][tj][v] - mn);
        lse[tj].l = lse[tj].l * __expf(lse[tj].m - mn) + su;
        lse[tj].m = mn;
        const int dt = target[tj] - f0;   // target among this lane's 4 x 4 features?
        if (dt >= 0 && dt < 32 && (dt & 4) == 0) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (dt == 8 * (v >> 2) + (v & 3)) ztarget[row] = acc[fi][tj][v];
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
    float* p = partials + ((size_t)bx * max_rows + row) * 2;
    p[0] = a.m; p[1] = a.l;
  }
}

__global__ void k_lmhead_score_merge(const float* __restrict__ partials, int max_rows, int n_groups,
                                     const int* __restrict__ n_rows_dev, const int* __restrict__ row_seq_pos, int T,
                                     float* __restrict__ out_logprobs) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= *n_rows_dev) return;
  LseAcc a; a.init();
  for (int s = 0; s < n_groups; ++s) {
    const float* p = partials + ((size_t)s * max_rows + row) * 2;
    a.merge(p[0], p[1]);
  }
  const float zt = partials[(size_t)max_rows * 2 * n_groups + row];
  out_logprobs[(size_t)row_seq_pos[2 * row] * T + row_seq_pos[2 * row + 1]] = zt - (a.m + logf(a.l));
}

hipError_t m_lmhead_score(const void* Xp, const void* Wp, int max_rows, const int* n_rows_dev, int V, int K,
                          const int* row_seq_pos, const int32_t* tokens, int T, float* partials, float* out_logprobs,
                          hipStream_t st) {
  if (max_rows == 0) return hipSuccess;
  if (V % 128 != 0 || K % 32 != 0) return hipErrorInvalidValue;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_lmhead_score, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int n_groups = score_groups(V);
  const hipError_t e = launch(KID_LMHEAD_SCORE, k_lmhead_score, dim3(big_grid(n_groups, (max_rows + 255) / 256)), dim3(256),
                              kBigLds, st, (const uint4*)Xp, (const uint4*)Wp, max_rows, n_rows_dev, V, K, row_seq_pos, tokens,
                              T, partials);
  if (e != hipSuccess) return e;
  return launch(KID_LMHEAD_SCORE_MERGE, k_lmhead_score_merge, dim3((max_rows + 255) / 256), dim3(256), 0, st, partials,
                max_rows, n_groups, n_rows_dev, row_seq_pos, T, out_logprobs);
}

// ---------------------------------------------------------------------------------------
// LM head for decode with many sequences (or a K too large for the 64-token kernel): the scoring
// GEMM's main loop with the sampler's epilogue, one (256 sequences x 128 vocabulary ids) tile per
// workgroup.  A lane turns its quads of consecutive vocabulary ids into perturbed scores (one Philox
// block per quad) and reduces, for each of its 4 sequences, (max, sum exp) and the best perturbed
// score.  partials: [V / 128][n_rows][5].
// ---------------------------------------------------------------------------------------
int m_lmhead_sample_big_groups(int V) { return V >> 7; }

__global__ void __launch_bounds__(256, 2) k_lmhead_sample_big(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp,
                                                              int n_rows, int V, int K, SampleParams sp,
                                                              float* __restrict__ partials) {
  extern __shared__ uint4 smem[];
  int ft, by;
  if (!big_raster(V >> 7, (n_rows + 255) >> 8, ft, by)) return;
  const int tok0 = by * 256;
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
  const int wf = wave & 1, wt = wave >> 1;
  f32x16 acc[2][4];
  big_mainloop(Xp, Wp, (n_rows + 31) >> 5, K >> 4, by * 8, ft * 4, smem, acc);
  resolve_sample_params(sp);
  const int step = *sp.step;
  const bool noisy = sp.temperature != 0.f;
  const float inv_t = noisy ? 1.0f / sp.temperature : 1.0f;
  wg_barrier();   // the ring is free: it carries the cross-wave merge
  float* red = (float*)smem;   // [2][256][5]
#pragma unroll
  for (int tj = 0; tj < 4; ++tj) {
    const int row_ = tok0 + wt * 128 + tj * 32 + (lane & 31);
    const int seq = (sp.slot_seq && row_ < n_rows) ? sp.slot_seq[row_] : row_;   // the noise is keyed on the sequence
    LseAcc lse;
    BestAcc best;
    lse.init();
    best.init();
#pragma unroll
    for (int fi = 0; fi < 2; ++fi) {
      float mt = acc[fi][tj][0];
#pragma unroll
      for (int v = 1; v < 16; ++v) mt = fmaxf(mt, acc[fi][tj][v]);
      const float mn = fmaxf(lse.m, mt);
      float su = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) su += __expf(acc[fi][tj][v] - mn);
      lse.l = lse.l * __expf(lse.m - mn) + su;
      lse.m = mn;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int v0 = ft * 128 + wf * 64 + fi * 32 + 8 * r + (lane >> 5) * 4;
        float gn[4] = {0.f, 0.f, 0.f, 0.f};
        if (noisy) gumbel4(sp.seed_lo, sp.seed_hi, (uint32_t)seq, (uint32_t)step, (uint32_t)(v0 >> 2), gn);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float z = acc[fi][tj][4 * r + j];
          const float y = noisy ? z * inv_t + gn[j] : z;
          if (y > best.y) { best.y = y; best.z = z; best.id = v0 + j; }   // ids ascend within a lane
        }
      }
    }
    // the two lane halves (fixed order); the two feature waves meet in LDS
    lse.merge(__shfl_xor(lse.m, 32, 64), __shfl_xor(lse.l, 32, 64));
    best.add(__shfl_xor(best.y, 32, 64), __shfl_xor(best.z, 32, 64), __shfl_xor(best.id, 32, 64));
    if (lane < 32) {
      float* p = red + ((size_t)wf * 256 + wt * 128 + tj * 32 + lane) * 5;
      p[0] = lse.m; p[1] = lse.l; p[2] = best.y; p[3] = best.z; ((int*)p)[4] = best.id;
    }
  }
  __syncthreads();
  const int row = tok0 + threadIdx.x;
  if (row < n_rows) {
    LseAcc a; a.init();
    BestAcc b; b.init();
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      const float* p = red + ((size_t)w * 256 + threadIdx.x) * 5;
      a.merge(p[0], p[1]);
      b.add(p[2], p[3], ((const int*)p)[4]);
    }
    float* p = partials + ((size_t)ft * n_rows + row) * 5;
    p[0] = a.m; p[1] = a.l; p[2] = b.y; p[3] = b.z; ((int*)p)[4] = b.id;
  }
}

hipError_t m_lmhead_sample_big(const void* Xp, const void* Wp, int n_rows, int V, int K, SampleParams sp, float* partials,
                               hipStream_t st) {
  if (n_rows <= 0 || V % 128 != 0 || K % 32 != 0) return hipErrorInvalidValue;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)k_lmhead_sample_big, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  return launch(KID_LMHEAD_SAMPLE, k_lmhead_sample_big, dim3(big_grid(V >> 7, (n_rows + 255) / 256)), dim3(256),
                kBigLds, st, (const uint4*)Xp, (const uint4*)Wp, n_rows, V, K, sp, partials);
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
// block-level synchronisation; waves never exchange data.  q (row-major [rows, Hq hd]), K, V and the
// probabilities are IEEE half; the output goes out as half in X32 order (the O projection's operand).
// ---------------------------------------------------------------------------------------
template <int HD, int HPW>
__global__ void __launch_bounds__(256, 2) k_flash_attention(const f16* __restrict__ q, RowMap rm, KVCache kv,
                                                         f16* __restrict__ out, int n_q_heads) {
  constexpr int KK = HD / 32, DT = HD / 16;
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
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
  const f16* kpool = (const f16*)kv.k;
  const f16* vpool = (const f16*)kv.v;
  const size_t page_elems = (size_t)hkv * kPageTokens * HD;
  // K / V fragments of a page pair; the next pair's are requested before the current one is multiplied (a third
  // register set, two pairs ahead, was measured at head dim 64: 238 against 223 us per launch at 64 x 768)
  Frag kf[2][KK], vf[DT], kn[2][KK], vn[DT];
  auto fetch = [&](int pp, Frag (&kd)[2][KK], Frag (&vd)[DT]) {
    const int pa = pt[2 * pp];
    const int pb = pt[min(2 * pp + 1, last_page)];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = lane & 15;
      const int ptok = 8 * (r >> 2) + 4 * t + (r & 3);   // key row r of score tile t
      const f16* kp = kpool + (size_t)(ptok < 16 ? pa : pb) * page_elems + ((size_t)kvh * kPageTokens + (ptok & 15)) * HD;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kd[t][kk].u = *(const uint4*)(kp + kk * 32 + grp * 8);
    }
    const f16* vp = vpool + (size_t)(grp < 2 ? pa : pb) * page_elems + (size_t)kvh * HD * kPageTokens + (grp & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vd[dt].u = *(const uint4*)(vp + (size_t)(dt * 16 + (lane & 15)) * kPageTokens);
  };
  fetch(0, kn, vn);
  for (int pp = 0; pp < npairs; ++pp) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[t][kk] = kn[t][kk];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[dt] = vn[dt];
    if (pp + 1 < npairs) fetch(pp + 1, kn, vn);
    const bool diag = pp * 32 + 31 > q0;   // some (query, key) of the pair is masked
#pragma unroll
    for (int h = 0; h < HPW; ++h) {
      if (h >= nh) continue;
      f32x4 sc[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) sc[t] = mfma16h(kf[t][kk], qf[h][kk], sc[t]);
      }
      // lane (query qcol, group grp) holds keys pp*32 + 8 grp + e, e = 4 t + j
      float p[8];   // raw scores; the softmax scale enters through the exponent's fma
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = sc[e >> 2][e & 3];
      if (diag) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (pp * 32 + 8 * grp + e > qpos) p[e] = -INFINITY;
      }
      float m_loc = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
      m_loc = max_xor16(m_loc);
      m_loc = max_xor32(m_loc);
      const float m_new = fmaxf(m_run[h], m_loc * scale2);   // finite: key 0 is visible to every query
      const float alpha = __builtin_amdgcn_exp2f(m_run[h] - m_new);   // exp2(-inf) = 0 on the first pair
      float psum = 0.f;
      Frag pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = __builtin_amdgcn_exp2f(fmaf(p[e], scale2, -m_new));
        psum += pe;
        pf.h[e] = (f16)pe;
      }
      l_run[h] = l_run[h] * alpha + psum;
      m_run[h] = m_new;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // the running max moved in some lane
        // the empty statement keeps this a branch: turned into selects, the 16 multiplies (and 16 selects) would run
        // for every pair, a quarter of the loop's vector-ALU work
        asm volatile("");
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int j = 0; j < 4; ++j) o[h][dt][j] *= alpha;
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[h][dt] = mfma16h(vf[dt], pf, o[h][dt]);
    }
  }
  if (q0 + qcol >= T) return;
#pragma unroll
  for (int h = 0; h < HPW; ++h) {
    if (h >= nh) continue;
    float l = l_run[h];
    l = sum_xor16(l);
    l = sum_xor32(l);
    const float inv = 1.0f / l;
    const int col0 = (kvh * rep + h0 + h) * HD + grp * 4;   // lane's 4 consecutive head dims, per 16-row tile
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      f16x4 ov;
#pragma unroll
      for (int j = 0; j < 4; ++j) ov[j] = from_f32<f16>(o[h][dt][j] * inv);
      const int col = col0 + dt * 16;
      *(f16x4*)(out + x32_chunk((int)row0 + qpos, col, (int)(qstride >> 4)) * 8 + (col & 4)) = ov;
    }
  }
}

hipError_t m_flash_attention(const void* q, RowMap rm, KVCache kv, void* out, int n_seq, int n_q_heads, hipStream_t st) {
  if (n_seq == 0) return hipSuccess;
  const int rep = n_q_heads / kv.n_kv_heads;
  const int nqb = (rm.T + 63) / 64;
  if (kv.head_dim == 64) {
    constexpr int HPW = 4;   // a 7-head group goes to two workgroups (4 + 3 heads): two waves per SIMD, which hide
                             // the softmax arithmetic, pay for the second read of K / V (2 heads each: slower again)
    dim3 grid(nqb, n_seq * kv.n_kv_heads, (rep + HPW - 1) / HPW);
    return launch(KID_FLASH_ATTN, k_flash_attention<64, HPW>, grid, dim3(256), 0, st, (const f16*)q, rm, kv, (f16*)out, n_q_heads);
  }
  if (kv.head_dim == 128) {
    constexpr int HPW = 2;
    dim3 grid(nqb, n_seq * kv.n_kv_heads, (rep + HPW - 1) / HPW);
    return launch(KID_FLASH_ATTN, k_flash_attention<128, HPW>, grid, dim3(256), 0, st, (const f16*)q, rm, kv, (f16*)out, n_q_heads);
  }
  return hipErrorInvalidValue;
}

}  // namespace sapo
