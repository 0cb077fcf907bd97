// The local policy update of a SAPO node (Algorithm 1, the PolicyGradient step; Sec. 4.2: GRPO without a
// KL term, asymmetric clipping, Adam with its default hyper-parameters): kernels, orchestration, C ABI.
//
// Values are fp32 on row-major buffers: master parameters, activations, gradients and the two Adam
// moments; the large GEMMs form their products from bf16 pieces on the matrix cores at fp32 accuracy
// (k_gemm_x3).  One update = forward pass over the whole training set with every layer's activations
// kept (HBM is large enough: about 80 KB per token and layer for the 0.5B shape), the clipped surrogate,
// the backward pass, one Adam step.  No atomics: every sum has a fixed order, so an update is
// reproducible bit for bit.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "surrogate.h"
#include "train.h"

using namespace sapo;

#define T_CK(expr)                                                                                     \
  do {                                                                                                 \
    hipError_t e__ = (expr);                                                                           \
    if (e__ != hipSuccess)                                                                             \
      return set_error(SAPO_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
  } while (0)

namespace {

// ---------------------------------------------------------------------------------------
// C[M, N] (ldc) = beta * C + op(A) op(B), fp32.  op(A) is M x K: A[m * lda + k], or A[k * lda + m] when
// TA; op(B) is K x N: B[k * ldb + n], or B[n * ldb + k] when TB.  64 x 64 tile per workgroup of 256
// threads, 4 x 4 outputs per thread, 16-deep k steps staged through LDS.  The three forms used:
//   y = x W^T (TA 0, TB 1), dx = dy W (0, 0), dW = dy^T x (1, 0).
// ---------------------------------------------------------------------------------------
constexpr int kTM = 64, kTN = 64, kTK = 16, kPitch = 68;

// Batched launches (blockIdx.z = batch b): with s = b / nh and h = b % nh the operands start at
// A + s a1 + h a2, B + s b1 + (h / bdiv) b2, C + s c1 + h c2 (elements).  nh = 1 and zeros: one GEMM.
struct Batch {
  int nh = 1, bdiv = 1;
  long a1 = 0, a2 = 0, b1 = 0, b2 = 0, c1 = 0, c2 = 0;
  int count = 1;
  // causal attention products (rows and columns are positions of one sequence): 1 = only output tiles with
  // column <= row are needed (scores, dP); 2 = op(A)[i][k] is zero for k > i, the k loop ends at the tile's last
  // row (P V, dS K); 3 = op(A)[j][k] is zero for k < j, the k loop starts at the tile's first row (dS^T Q, P^T dO)
  int causal = 0;
  // Segmented contraction (MFMA kernel only): K consists of K / kseg segments of kseg (a multiple of 16); segment g
  // reads op(A) from A + g sega and op(B) from B + g segb, indexed by k - g kseg.  With causal = 3 the skipped start
  // applies to every segment.  Used to add the query heads of a group up inside one GEMM, in head order.
  int kseg = 0;
  long sega = 0, segb = 0;
};
// Tile of a 1-D launch of nx * ny workgroups.  Workgroup ids are dealt round-robin to the 8 XCDs (each with its
// own L2), so XCD x = id % 8 takes the contiguous tile range [x per, (x + 1) per) and walks it in panels of 8
// tile rows, column by column: the ~100 workgroups an XCD runs at once then share 8 row blocks and a dozen
// column blocks through its L2 instead of streaming every block from the memory side.
__device__ __forceinline__ bool raster_tile(int nx, int ny, int& tx, int& ty) {
  const int nt = nx * ny, per = (nt + 7) >> 3;
  const int j = blockIdx.x >> 3, t = (blockIdx.x & 7) * per + j;
  if (j >= per || t >= nt) return false;
  const int panel = t / (8 * nx), w = t - panel * 8 * nx;
  const int rows = min(8, ny - panel * 8);
  ty = panel * 8 + w % rows;
  tx = w / rows;
  return true;
}
inline unsigned raster_grid(int nx, int ny) { return (unsigned)(((long)nx * ny + 7) / 8 * 8); }

__device__ __forceinline__ void batch_offsets(const Batch& bt, const float* __restrict__& A, const float* __restrict__& B,
                                              float* __restrict__& C) {
  const int b = blockIdx.z, s = b / bt.nh, h = b % bt.nh;
  A += s * bt.a1 + h * bt.a2;
  B += s * bt.b1 + (h / bt.bdiv) * bt.b2;
  C += s * bt.c1 + h * bt.c2;
}

template <int TA, int TB>
__global__ void __launch_bounds__(256) k_sgemm(const float* __restrict__ A, int lda, const float* __restrict__ B, int ldb,
                                               float* __restrict__ C, int ldc, int M, int N, int K, float beta, Batch bt) {
  __shared__ __align__(16) float As[kTK][kPitch];
  __shared__ __align__(16) float Bs[kTK][kPitch];
  batch_offsets(bt, A, B, C);
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * kTM, n0 = blockIdx.x * kTN;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += kTK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + 256 * i;
      {
        const int mm = TA ? (e & 63) : (e >> 4), kk = TA ? (e >> 6) : (e & 15);
        const int m = m0 + mm, k = k0 + kk;
        float v = 0.f;
        if (m < M && k < K) v = TA ? A[(size_t)k * lda + m] : A[(size_t)m * lda + k];
        As[kk][mm] = v;
      }
      {
        const int nn = TB ? (e >> 4) : (e & 63), kk = TB ? (e & 15) : (e >> 6);
        const int n = n0 + nn, k = k0 + kk;
        float v = 0.f;
        if (n < N && k < K) v = TB ? B[(size_t)n * ldb + k] : B[(size_t)k * ldb + n];
        Bs[kk][nn] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kTK; ++kk) {
      const float4 a = *(const float4*)&As[kk][ty * 4];
      const float4 b = *(const float4*)&Bs[kk][tx * 4];
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float* c = C + (size_t)m * ldc + n;
      *c = (beta != 0.f) ? fmaf(beta, *c, acc[i][j]) : acc[i][j];
    }
  }
}

// The same contraction on the matrix cores (v_mfma_f32_32x32x2_f32: fp32 operands, fp32 accumulation), for
// operands whose sizes and leading dimensions are multiples of 4 and whose bases are 16-byte aligned.
// 128 x 128 tile per workgroup, 4 waves of 64 x 64 (2 x 2 MFMA tiles), 16-deep k steps, two LDS buffers: the
// next step's operands are fetched into registers while the current step is multiplied.  LDS rows are k,
// 160 floats apart, so the two k rows a wave reads at once fall into disjoint banks.
constexpr int kGM = 128, kGK = 16, kGP = 160;
typedef float f32x16_t __attribute__((ext_vector_type(16)));

template <int TRANS>   // TRANS 0: src[row * ld + k] (k contiguous); 1: src[k * ld + row] (row contiguous)
__device__ __forceinline__ void gemm_fetch(const float* __restrict__ src, int ld, int row0, int n_rows, int k0, int K,
                                           float4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = threadIdx.x + 256 * i;
    r[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (TRANS == 0) {
      const int row = row0 + (e >> 2), k = k0 + (e & 3) * 4;
      if (row < n_rows && k < K) r[i] = *(const float4*)(src + (size_t)row * ld + k);
    } else {
      const int k = k0 + (e >> 5), row = row0 + (e & 31) * 4;
      if (row < n_rows && k < K) r[i] = *(const float4*)(src + (size_t)k * ld + row);
    }
  }
}
template <int TRANS>
__device__ __forceinline__ void gemm_stage(float (*buf)[kGP], const float4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = threadIdx.x + 256 * i;
    if (TRANS == 0) {
      const int row = e >> 2, k = (e & 3) * 4;
      buf[k][row] = r[i].x; buf[k + 1][row] = r[i].y; buf[k + 2][row] = r[i].z; buf[k + 3][row] = r[i].w;
    } else {
      *(float4*)&buf[e >> 5][(e & 31) * 4] = r[i];
    }
  }
}

template <int TA, int TB, int NARROW>   // NARROW: N <= 64, the four waves stack along M (32 rows x 64 columns each)
__global__ void __launch_bounds__(256) k_sgemm_mfma(const float* __restrict__ A, int lda, const float* __restrict__ B, int ldb,
                                                    float* __restrict__ C, int ldc, int M, int N, int K, float beta,
                                                    Batch bt) {
  __shared__ __align__(16) float As[2][kGK][kGP];
  __shared__ __align__(16) float Bs[2][kGK][kGP];
  batch_offsets(bt, A, B, C);
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
  int tx, ty;
  if (!raster_tile((N + kGM - 1) / kGM, (M + kGM - 1) / kGM, tx, ty)) return;
  const int m0 = ty * kGM, n0 = tx * kGM;
  constexpr int MI = NARROW ? 1 : 2;
  const int wm = NARROW ? wave * 32 : (wave >> 1) * 64, wn = NARROW ? 0 : (wave & 1) * 64;
  f32x16_t acc[MI][2];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  if (bt.causal == 1 && n0 > m0 + kGM - 1) return;   // the whole tile lies above the diagonal
  int t_begin = 0, nk = (K + kGK - 1) / kGK;
  if (bt.causal == 2) nk = min(nk, (m0 + kGM + kGK - 1) / kGK);
  if (bt.causal == 3) t_begin = min(m0 / kGK, nk - 1);
  // segmented contraction: step u is step seg_skip + u % per of segment u / per
  const int seg_steps = bt.kseg > 0 ? bt.kseg / kGK : 0;
  const int seg_skip = (seg_steps && bt.causal == 3) ? min(m0 / kGK, seg_steps - 1) : 0;
  const int per = seg_steps - seg_skip;
  if (seg_steps) { t_begin = 0; nk = (K / bt.kseg) * per; }
  float4 ra[2], rb[2];
  // op(A) rows are m: A is "k contiguous" unless TA; op(B) rows are n: B is "k contiguous" when TB
  auto fetch = [&](int u) {
    const float* Ag = A;
    const float* Bg = B;
    int k0 = u * kGK, Kb = K;
    if (seg_steps) {
      const int g = u / per;
      k0 = (seg_skip + u - g * per) * kGK;
      Ag += g * bt.sega;
      Bg += g * bt.segb;
      Kb = bt.kseg;
    }
    gemm_fetch<TA>(Ag, lda, m0, M, k0, Kb, ra);
    gemm_fetch<TB ? 0 : 1>(Bg, ldb, n0, N, k0, Kb, rb);
  };
  fetch(t_begin);
  gemm_stage<TA>(As[t_begin & 1], ra);
  gemm_stage<TB ? 0 : 1>(Bs[t_begin & 1], rb);
  __syncthreads();
  for (int t = t_begin; t < nk; ++t) {
    const int cur = t & 1;
    if (t + 1 < nk) fetch(t + 1);
#pragma unroll
    for (int kk = 0; kk < kGK; kk += 2) {
      const int kr = kk + (lane >> 5), c = lane & 31;
      const float b0 = Bs[cur][kr][wn + c], b1 = Bs[cur][kr][wn + 32 + c];
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const float a = As[cur][kr][wm + i * 32 + c];
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[i][0], 0, 0, 0);
        acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[i][1], 0, 0, 0);
      }
    }
    if (t + 1 < nk) {
      gemm_stage<TA>(As[cur ^ 1], ra);
      gemm_stage<TB ? 0 : 1>(Bs[cur ^ 1], rb);
    }
    __syncthreads();
  }
  // accumulator v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of the 32 x 32 tile
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      if (n >= N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (m >= M) continue;
        float* c = C + (size_t)m * ldc + n;
        *c = (beta != 0.f) ? fmaf(beta, *c, acc[i][j][v]) : acc[i][j][v];
      }
    }
}

// ---------------------------------------------------------------------------------------
// The large GEMMs at fp32 accuracy on the bf16 matrix cores.  An fp32 value is the exact sum of three bf16
// values (its 24-bit mantissa cut into three 8-bit pieces: hi, mid, lo); a product a b is taken as the six
// partial products of weight >= 2^-16 (hi hi, hi mid, mid hi, hi lo, lo hi, mid mid), each exact in fp32,
// the three dropped ones being below 2^-23 of the product: the rounding of an fp32 multiply.  Six
// v_mfma_f32_32x32x16_bf16 (32 cycles each) do the work of sixteen v_mfma_f32_32x32x2_f32 (64 cycles each).
// With one piece the same kernels are a plain bf16 GEMM with fp32 accumulation (the value rounded to nearest).
// With two pieces (the value rounded to bf16, then the exact remainder rounded to bf16: 16 significant bits) the
// three products hi hi, hi mid, mid hi are taken: what is dropped is below 2^-16 of a product and of either sign,
// at half the matrix-core work of the six-product form.
//
// Operands are cut once per GEMM by k_pack_x3 into the order a workgroup stages them in: for every block of
// 128 rows and every 16-k step, [piece][k half][row] entries of 8 bf16 (16 bytes): one contiguous 2 KB x
// pieces x 2 run per step, and the LDS image needs no rearrangement.  Rows and k are zero-padded to the
// blocks.  "Rows" are the M side of op(A) or the N side of op(B); k is the contraction.
// ---------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
// 16-byte entries as a plain vector type: with HIP's uint4 struct the compiler kept the kernel's prefetch registers
// in scratch memory (every load waited for at once, then re-read), 2.7x slower
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
union Frag8 { u32x4_t u; bf16x8_t v; };

__device__ __forceinline__ void split3(float x, uint32_t& hi, uint32_t& mid, uint32_t& lo) {   // bf16 bits in the high halves
  hi = __float_as_uint(x) & 0xFFFF0000u;
  const float r = x - __uint_as_float(hi);
  mid = __float_as_uint(r) & 0xFFFF0000u;
  const float r2 = r - __uint_as_float(mid);
  lo = __float_as_uint(r2) & 0xFFFF0000u;
}
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | b; }   // a low half, b high half

// entry (16 bytes) of (piece, row, k / 8) in a packed operand with KB = padded K / 16 steps
__device__ __forceinline__ size_t x3_entry(int NP, int KB, int piece, int row, int k8) {
  return ((((size_t)(row >> 7) * KB + (k8 >> 1)) * NP + piece) * 2 + (k8 & 1)) * 128 + (row & 127);
}
__device__ __forceinline__ void x3_store(uint4* __restrict__ dst, int NP, int KB, int row, int k8, const float (&x)[8]) {
  uint32_t p[3][8];
#pragma unroll
  for (int j = 0; j < 8; ++j) split3(x[j], p[0][j], p[1][j], p[2][j]);
  if (NP < 3) {   // one or two pieces are roundings to nearest even (of the value, then of what is left), not bit fields
    auto rne = [](float f) { const uint32_t u = __float_as_uint(f); return (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u; };
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p[0][j] = rne(x[j]);
      p[1][j] = rne(x[j] - __uint_as_float(p[0][j]));
    }
  }
  for (int pc = 0; pc < NP; ++pc)
    dst[x3_entry(NP, KB, pc, row, k8)] = make_uint4(pack_hi(p[pc][0], p[pc][1]), pack_hi(p[pc][2], p[pc][3]),
                                                    pack_hi(p[pc][4], p[pc][5]), pack_hi(p[pc][6], p[pc][7]));
}
// src[row * ld + k]: one workgroup per (block of 128 rows, 8 k steps); thread (row, k half) reads 8 consecutive
// k per step, so a row is read in 64-byte runs and every piece of a step goes out as two 2 KB runs
__global__ void __launch_bounds__(256) k_pack_x3(const float* __restrict__ src, int ld, int rows, int K, int /*rows_pad*/, int KB,
                                                 int NP, uint4* __restrict__ dst) {
  const int row = blockIdx.x * 128 + (threadIdx.x >> 1), kh = threadIdx.x & 1;
  const float* rp = src + (size_t)row * ld;
  const bool vec = ((ld & 3) == 0) && ((((uintptr_t)src) & 15) == 0);
  for (int kb = blockIdx.y * 8; kb < min(KB, blockIdx.y * 8 + 8); ++kb) {
    const int k0 = kb * 16 + kh * 8;
    float x[8];
    if (row < rows && k0 + 8 <= K && vec) {
      const float4 a = *(const float4*)(rp + k0), b = *(const float4*)(rp + k0 + 4);
      x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = (row < rows && k0 + j < K) ? rp[k0 + j] : 0.f;
    }
    x3_store(dst, NP, KB, row, kb * 2 + kh, x);
  }
}
// src[k * ld + row] (rows contiguous): 64 rows x 64 k per workgroup through LDS
__global__ void __launch_bounds__(256) k_pack_x3_t(const float* __restrict__ src, int ld, int rows, int K, int rows_pad, int KB,
                                                   int NP, uint4* __restrict__ dst) {
  __shared__ float tile[64][65];
  const int r0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
  for (int e = threadIdx.x; e < 64 * 64; e += 256) {
    const int kk = e >> 6, rr = e & 63;
    const int k = k0 + kk, row = r0 + rr;
    tile[kk][rr] = (row < rows && k < K) ? src[(size_t)k * ld + row] : 0.f;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 8; e += 256) {
    const int rr = e & 63, kq = e >> 6;           // 8 groups of 8 k
    const int row = r0 + rr, k8 = (k0 >> 3) + kq;
    if (row >= rows_pad || k8 >= KB * 2) continue;
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = tile[kq * 8 + j][rr];
    x3_store(dst, NP, KB, row, k8, x);
  }
}

// RB = row blocks of 128 per tile: 1 (128 x 128, three workgroups per CU) or 2 (256 x 128 for outputs with many
// tiles: each wave 128 x 64, two workgroups per CU, a quarter less traffic per flop on both the L2 and the LDS side)
template <int NP, int RB>
__global__ void __launch_bounds__(256, RB == 2 ? 2 : 3) k_gemm_x3(const u32x4_t* __restrict__ Ap, const u32x4_t* __restrict__ Bp,
                                                                  float* __restrict__ C, int ldc, int M, int N, int KB, float beta,
                                                                  int kb_split, size_t c_split) {
  constexpr int E = NP * 256;                 // 16-byte entries per row block, operand and k step
  constexpr int MI = 2 * RB;                  // 32-row MFMA tiles per wave
  __shared__ u32x4_t As[2][RB * E];
  __shared__ u32x4_t Bs[2][E];
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63;
  int tx, ty;
  const int n_rb = (M + kGM - 1) / kGM;       // row blocks of the packed operand
  if (!raster_tile((N + kGM - 1) / kGM, (n_rb + RB - 1) / RB, tx, ty)) return;
  const int m0 = ty * kGM * RB, n0 = tx * kGM;
  const int wm = (wave >> 1) * 64 * RB, wn = (wave & 1) * 64;
  const u32x4_t* ap[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r)   // a tile's last row block may not exist: it repeats the previous one and is not stored
    ap[r] = Ap + (size_t)min(ty * RB + r, n_rb - 1) * KB * E + threadIdx.x;
  const u32x4_t* bp = Bp + (size_t)tx * KB * E + threadIdx.x;
  f32x16_t acc[MI][2];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // blockIdx.z takes the k steps [z kb_split, (z + 1) kb_split) and writes its own copy of C (split weight gradients)
  const int t0 = blockIdx.z * kb_split, t1 = min(KB, t0 + kb_split);
  C += (size_t)blockIdx.z * c_split;
  u32x4_t ra[RB][NP], rb[NP];
#pragma unroll
  for (int pc = 0; pc < NP; ++pc) {
#pragma unroll
    for (int r = 0; r < RB; ++r) ra[r][pc] = ap[r][(size_t)t0 * E + pc * 256];
    rb[pc] = bp[(size_t)t0 * E + pc * 256];
  }
#pragma unroll
  for (int pc = 0; pc < NP; ++pc) {
#pragma unroll
    for (int r = 0; r < RB; ++r) As[0][r * E + pc * 256 + threadIdx.x] = ra[r][pc];
    Bs[0][pc * 256 + threadIdx.x] = rb[pc];
  }
  __syncthreads();
  const int kh = lane >> 5, c = lane & 31;
  for (int t = t0; t < t1; ++t) {
    const int cur = (t - t0) & 1;
    if (t + 1 < t1) {
#pragma unroll
      for (int pc = 0; pc < NP; ++pc) {
#pragma unroll
        for (int r = 0; r < RB; ++r) ra[r][pc] = ap[r][(size_t)(t + 1) * E + pc * 256];
        rb[pc] = bp[(size_t)(t + 1) * E + pc * 256];
      }
    }
    Frag8 b[2][NP];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int pc = 0; pc < NP; ++pc) b[j][pc].u = Bs[cur][(pc * 2 + kh) * 128 + wn + j * 32 + c];
    // smallest partial products first: (hi lo), (lo hi), (mid mid), (hi mid), (mid hi), (hi hi); two pieces take the
    // last three, one piece the last
    constexpr int n_terms = NP == 3 ? 6 : NP == 2 ? 3 : 1;
    constexpr int pa[6] = {0, 2, 1, 0, 1, 0}, pb[6] = {2, 0, 1, 1, 0, 0};
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      Frag8 a[NP];
      const int row = wm + i * 32 + c;        // within the tile: row block row >> 7
#pragma unroll
      for (int pc = 0; pc < NP; ++pc) a[pc].u = As[cur][(row >> 7) * E + (pc * 2 + kh) * 128 + (row & 127)];
#pragma unroll
      for (int term = 6 - n_terms; term < 6; ++term)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pa[term]].v, b[j][pb[term]].v, acc[i][j], 0, 0, 0);
    }
    if (t + 1 < t1) {
#pragma unroll
      for (int pc = 0; pc < NP; ++pc) {
#pragma unroll
        for (int r = 0; r < RB; ++r) As[cur ^ 1][r * E + pc * 256 + threadIdx.x] = ra[r][pc];
        Bs[cur ^ 1][pc * 256 + threadIdx.x] = rb[pc];
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      if (n >= N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (m >= M) continue;
        float* cp = C + (size_t)m * ldc + n;
        *cp = (beta != 0.f) ? fmaf(beta, *cp, acc[i][j][v]) : acc[i][j][v];
      }
    }
}

// One operand of a packed GEMM: `rows` x K values at src[row * ld + k], or src[k * ld + row] when `trans`.
struct X3Op { const float* src; int ld, rows, K; bool trans; };
inline size_t x3_pack_bytes(int NP, size_t rows, size_t K) {
  return ((rows + 127) / 128 * 128) * ((K + 15) / 16 * 16) * 2 * NP;
}
struct X3Bufs { void* a; void* b; size_t a_cap, b_cap; int NP; float* parts; size_t parts_cap; };
constexpr int kMaxSplits = 16;
__global__ void k_sum_parts(const float* __restrict__ part, int n_part, size_t n, float beta, float* __restrict__ out);

hipError_t x3_pack(const X3Op& op, void* dst, size_t cap, int NP, hipStream_t st) {
  if (x3_pack_bytes(NP, op.rows, op.K) > cap) return hipErrorInvalidValue;
  const int rows_pad = (op.rows + 127) / 128 * 128, KB = (op.K + 15) / 16;
  if (!op.trans)
    return launch(KID_MISC, k_pack_x3, dim3(rows_pad / 128, (KB + 7) / 8), dim3(256), 0, st, op.src, op.ld, op.rows, op.K, rows_pad,
                  KB, NP, (uint4*)dst);
  return launch(KID_MISC, k_pack_x3_t, dim3(rows_pad / 64, (KB * 16 + 63) / 64), dim3(256), 0, st, op.src, op.ld, op.rows, op.K,
                rows_pad, KB, NP, (uint4*)dst);
}
// C[M, N] = beta C + op(A) op(B)^T-style product of two operands given row-wise over the same K
hipError_t gemm_x3(const X3Op& A, const X3Op& B, float* C, int ldc, float beta, const X3Bufs& bufs, hipStream_t st,
                   bool split_ok = false, const void* a_packed = nullptr, const void* b_packed = nullptr) {
  if (A.K != B.K || A.rows <= 0 || B.rows <= 0 || A.K <= 0) return hipErrorInvalidValue;
  hipError_t e;
  // an operand packed earlier (a_packed / b_packed) is used as it is
  if (!a_packed && (e = x3_pack(A, bufs.a, bufs.a_cap, bufs.NP, st)) != hipSuccess) return e;
  if (!b_packed && (e = x3_pack(B, bufs.b, bufs.b_cap, bufs.NP, st)) != hipSuccess) return e;
  const u32x4_t* pa_ = (const u32x4_t*)(a_packed ? a_packed : bufs.a);
  const u32x4_t* pb_ = (const u32x4_t*)(b_packed ? b_packed : bufs.b);
  const int KB = (A.K + 15) / 16;
  const int gnx = (B.rows + kGM - 1) / kGM, gny = (A.rows + kGM - 1) / kGM;
  // 256-row tiles when the output still has plenty of them
  const int RB = (gnx >= 32 && (long)gnx * ((gny + 1) / 2) >= 512) ? 2 : 1;
  const int gty = (gny + RB - 1) / RB;
  dim3 grid(raster_grid(gnx, gty), 1);
  // A long contraction whose output tiles do not fill the workgroups in flight (weight gradients: 49 .. 532 tiles
  // against 768 resident workgroups, or a last round that is mostly empty): the k steps are split into parts, each
  // part writes its own product and k_sum_parts adds them in part order.  The number of parts is the one whose
  // rounds of resident workgroups are fullest; more parts must buy at least 4 % (they cost a pass over the output).
  const long tiles = (long)gnx * gty;
  int splits = 1;
  if (split_ok && ldc == B.rows) {
    const long slots = RB == 2 ? 512 : 768;
    double best = 0.0;
    for (int s_ = 1; s_ <= kMaxSplits; ++s_) {
      if (s_ > 1 && (KB / s_ < 16 || (size_t)s_ * A.rows * B.rows > bufs.parts_cap)) break;
      const long units = tiles * s_;
      const double fill = (double)units / (double)((units + slots - 1) / slots * slots);
      if (fill > best + 0.04) { best = fill; splits = s_; }
    }
  }
  const int kbs = (KB + splits - 1) / splits;
  splits = (KB + kbs - 1) / kbs;
  grid.z = splits;
  float* out = splits > 1 ? bufs.parts : C;
  const size_t c_split = splits > 1 ? (size_t)A.rows * B.rows : 0;
  const float b_ = splits > 1 ? 0.f : beta;
  auto go = [&](auto kernel) {
    return launch(KID_GEMM_GENERIC, kernel, grid, dim3(256), 0, st, pa_, pb_, out, ldc, A.rows, B.rows, KB, b_, kbs, c_split);
  };
  if (bufs.NP == 3) e = RB == 2 ? go(k_gemm_x3<3, 2>) : go(k_gemm_x3<3, 1>);
  else if (bufs.NP == 2) e = RB == 2 ? go(k_gemm_x3<2, 2>) : go(k_gemm_x3<2, 1>);
  else e = RB == 2 ? go(k_gemm_x3<1, 2>) : go(k_gemm_x3<1, 1>);
  if (e != hipSuccess || splits == 1) return e;
  const size_t n = (size_t)A.rows * B.rows;
  return launch(KID_MISC, k_sum_parts, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const float*)bufs.parts, splits, n, beta,
                C);
}

template <int TA, int TB>
hipError_t sgemm(const float* A, int lda, const float* B, int ldb, float* C, int ldc, int M, int N, int K, float beta,
                 hipStream_t st, const Batch& bt = Batch()) {
  if (M <= 0 || N <= 0 || K <= 0 || bt.count <= 0 || bt.count > 65535) return hipErrorInvalidValue;
  if (bt.kseg > 0 && (bt.kseg % kGK != 0 || K % bt.kseg != 0)) return hipErrorInvalidValue;
  const long strides = bt.a1 | bt.a2 | bt.b1 | bt.b2 | bt.sega | bt.segb;
  const bool aligned = ((M | N | K | lda | ldb) & 3) == 0 && (strides & 3) == 0 && (((uintptr_t)A | (uintptr_t)B) & 15) == 0;
  if (aligned && (long)M * N * bt.count >= 128 * 128) {
    const dim3 grid(raster_grid((N + kGM - 1) / kGM, (M + kGM - 1) / kGM), 1, bt.count);
    if (N <= 64)
      return launch(KID_GEMM_GENERIC, k_sgemm_mfma<TA, TB, 1>, grid, dim3(256), 0, st, A, lda, B, ldb, C, ldc, M, N, K, beta, bt);
    return launch(KID_GEMM_GENERIC, k_sgemm_mfma<TA, TB, 0>, grid, dim3(256), 0, st, A, lda, B, ldb, C, ldc, M, N, K, beta, bt);
  }
  if (bt.kseg > 0) return hipErrorInvalidValue;   // the vector-ALU kernel has no segmented contraction
  return launch(KID_GEMM_GENERIC, k_sgemm<TA, TB>, dim3((N + kTN - 1) / kTN, (M + kTM - 1) / kTM, bt.count), dim3(256), 0, st, A,
                lda, B, ldb, C, ldc, M, N, K, beta, bt);
}

__device__ __forceinline__ float block_sum256(float v, float* red) {
  v = wave_reduce_sum(v);
  __syncthreads();   // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ float block_max256(float v, float* red) {
  v = wave_reduce_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// ---------------------------------------------------------------------------------------
// storage type <-> fp32 masters
// ---------------------------------------------------------------------------------------
__global__ void k_bf16_to_f32(const bf16* __restrict__ src, float* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = (float)src[i];
}
__global__ void k_f32_to_bf16(const float* __restrict__ src, bf16* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = from_f32<bf16>(src[i]);   // round to nearest even
}

// ---------------------------------------------------------------------------------------
// forward pieces
// ---------------------------------------------------------------------------------------
// token ids outside [0, V) are clamped into it (a caller's mistake must not become a wild access)
__device__ __forceinline__ int clamp_token(int t, int V) { return min(max(t, 0), V - 1); }

__global__ void __launch_bounds__(256) k_embed_rows(const int32_t* __restrict__ tokens, const float* __restrict__ embed,
                                                    float* __restrict__ h, int d, int V) {
  const size_t m = blockIdx.x;
  const float* src = embed + (size_t)clamp_token(tokens[m], V) * d;
  for (int i = threadIdx.x; i < d; i += 256) h[m * d + i] = src[i];
}

// xn = h * rstd * gain, rstd = 1 / sqrt(mean(h^2) + eps); one workgroup per row
__global__ void __launch_bounds__(256) k_rmsnorm_fwd(const float* __restrict__ h, const float* __restrict__ gain, float eps,
                                                     int d, float* __restrict__ xn, float* __restrict__ rstd) {
  __shared__ float red[4];
  const size_t m = blockIdx.x;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float v = h[m * d + i]; ss = fmaf(v, v, ss); }
  ss = block_sum256(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  if (threadIdx.x == 0) rstd[m] = r;
  for (int i = threadIdx.x; i < d; i += 256) xn[m * d + i] = h[m * d + i] * r * gain[i];
}

// Rotary embedding in place on the query and key heads of qkv[M, (Hq + 2 Hkv) hd]; position = row % T.
// dir = +1 rotates by the angle, -1 by its negative (the transpose: what the backward pass applies).
__global__ void k_rope(float* __restrict__ qkv, const float2* __restrict__ rope, int T, int n_rot_heads, int hd, int row_len,
                       float dir, size_t total) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int half = hd >> 1;
  const int i = (int)(idx % half);
  const int head = (int)((idx / half) % n_rot_heads);
  const size_t m = idx / ((size_t)half * n_rot_heads);
  const float2 cs = rope[(size_t)(m % T) * half + i];
  float* p = qkv + m * row_len + (size_t)head * hd + i;
  const float x1 = p[0], x2 = p[half], s = cs.y * dir;
  p[0] = x1 * cs.x - x2 * s;
  p[half] = x2 * cs.x + x1 * s;
}

// Causal grouped-query attention through batched GEMMs: scores[s, h] = Q_h K^T (T x T per sequence and
// query head), the row kernels below, out = P V.  Row r = (s * Hq + h) * T + i of the score buffer.
// k_softmax_causal: in place, p_ij = softmax_j(scale * s_ij) over j <= i, 0 for j > i; lse[r] = log sum_j exp(scale * s_ij).
__global__ void __launch_bounds__(64) k_softmax_causal(float* __restrict__ sc, float* __restrict__ lse, int T, float scale) {
  const size_t r = blockIdx.x;
  const int i = (int)(r % T), lane = threadIdx.x;
  float* row = sc + r * T;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) mx = fmaxf(mx, row[j] * scale);
  mx = wave_reduce_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= i; j += 64) sum += expf(row[j] * scale - mx);
  sum = wave_reduce_sum(sum);
  const float l = mx + logf(sum);
  if (lane == 0) lse[r] = l;
  for (int j = lane; j < T; j += 64) row[j] = (j <= i) ? expf(row[j] * scale - l) : 0.f;
}
// the same probabilities from kept log-sum-exps (backward pass): p_ij = exp(scale * s_ij - lse[r]), 0 for j > i
__global__ void k_probs_from_lse(float* __restrict__ sc, const float* __restrict__ lse, int T, float scale, size_t total) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const size_t r = idx / T;
  const int j = (int)(idx % T), i = (int)(r % T);
  sc[idx] = (j <= i) ? expf(sc[idx] * scale - lse[r]) : 0.f;
}

// act = silu(gate) * up from gu[M, 2F] (gate columns first)
__global__ void k_swiglu_fwd(const float* __restrict__ gu, float* __restrict__ act, int F, size_t total) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const size_t m = idx / F;
  const int f = (int)(idx % F);
  const float g = gu[m * 2 * F + f], u = gu[m * 2 * F + F + f];
  act[idx] = g / (1.0f + expf(-g)) * u;
}

// ---------------------------------------------------------------------------------------
// LM head rows.  Row r = (s, t) of the final-normed states predicts tokens[s, t + 1].  One workgroup per row
// of a chunk of logits: log-sum-exp, logp_new[s, t + 1] = z[target] - lse, the token's surrogate gradient
// w = d loss / d logp (it needs only this token's log-probs, its sequence's advantage and the number of
// masked tokens), then in place  logits <- d loss / d logits = w (onehot(target) - softmax).
// Rows whose target is not masked, and the last row of every sequence, become zero.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_count_mask(const uint8_t* __restrict__ mask, size_t n, long long* __restrict__ out) {
  __shared__ int part[256];
  int c = 0;
  for (size_t i = threadIdx.x; i < n; i += 256) c += mask[i] != 0;
  part[threadIdx.x] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    long long t = 0;
    for (int j = 0; j < 256; ++j) t += part[j];
    *out = t;
  }
}
// Row k of `logits` belongs to row r = rows[k] of the batch (position r % T of sequence r / T), which predicts the
// masked token at r + 1 (the list holds exactly those rows).  In place: logits -> d loss / d logits.
__global__ void __launch_bounds__(256) k_logp_dlogits(float* __restrict__ logits, int V, const int* __restrict__ rows, int T,
                                                      const int32_t* __restrict__ tokens, const uint8_t* __restrict__ mask,
                                                      const float* __restrict__ logp_old, const float* __restrict__ adv,
                                                      float eps_low, float eps_high, const long long* __restrict__ n_masked,
                                                      float* __restrict__ logp_new) {
  __shared__ float red[4];
  const int r = rows[blockIdx.x];
  const int t = r % T;
  float* z = logits + (size_t)blockIdx.x * V;
  if (t == T - 1 || !mask[r + 1]) {   // not in a well-formed list; uniform over the workgroup
    for (int v = threadIdx.x; v < V; v += 256) z[v] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 256) mx = fmaxf(mx, z[v]);
  mx = block_max256(mx, red);
  float sum = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) sum += expf(z[v] - mx);
  sum = block_sum256(sum, red);
  const float l = mx + logf(sum);
  const int target = clamp_token(tokens[r + 1], V);
  const float lp = z[target] - l;
  float rho; bool active;
  const float a = adv[r / T];
  surrogate_term(lp, logp_old[r + 1], a, eps_low, eps_high, rho, active);
  const float w = surrogate_dlogp(a, rho, active, *n_masked);
  __syncthreads();   // every thread has read z[target]
  if (threadIdx.x == 0) logp_new[r + 1] = lp;
  for (int v = threadIdx.x; v < V; v += 256) z[v] = (w == 0.f) ? 0.f : w * ((v == target ? 1.f : 0.f) - expf(z[v] - l));
}

// dst[k] = src[rows[k]] (gather) or dst[rows[k]] = src[k] (scatter): rows of d floats, one workgroup per listed row
__global__ void __launch_bounds__(256) k_move_rows(const float* __restrict__ src, const int* __restrict__ rows, int d, int scatter,
                                                   float* __restrict__ dst) {
  const size_t k = blockIdx.x, r = (size_t)rows[blockIdx.x];
  const float* a = src + (scatter ? k : r) * d;
  float* b = dst + (scatter ? r : k) * d;
  for (int i = threadIdx.x; i < d; i += 256) b[i] = a[i];
}
// out = (beta ? out : 0) + sum over the parts, in part order
__global__ void k_sum_parts(const float* __restrict__ part, int n_part, size_t n, float beta, float* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = beta != 0.f ? beta * out[i] : 0.f;
  for (int p = 0; p < n_part; ++p) s += part[(size_t)p * n + i];
  out[i] = s;
}

// ---------------------------------------------------------------------------------------
// backward pieces
// ---------------------------------------------------------------------------------------
// RMSNorm: dh (+)= rstd * gain * dxn - rstd^3 * h * mean_j(dxn_j gain_j h_j); one workgroup per row.
__global__ void __launch_bounds__(256) k_rmsnorm_bwd(const float* __restrict__ dxn, const float* __restrict__ h,
                                                     const float* __restrict__ rstd, const float* __restrict__ gain, int d,
                                                     float* __restrict__ dh, int accumulate) {
  __shared__ float red[4];
  const size_t m = blockIdx.x;
  float dot = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) dot = fmaf(dxn[m * d + i] * gain[i], h[m * d + i], dot);
  dot = block_sum256(dot, red);
  const float r = rstd[m];
  const float c = r * r * r * dot / (float)d;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float g = r * gain[i] * dxn[m * d + i] - c * h[m * d + i];
    dh[m * d + i] = accumulate ? dh[m * d + i] + g : g;
  }
}
// d gain_i = sum_m dxn[m, i] h[m, i] rstd[m]: partial sums over blocks of 256 rows, then over the blocks in order
__global__ void __launch_bounds__(256) k_gain_grad_partial(const float* __restrict__ dxn, const float* __restrict__ h,
                                                           const float* __restrict__ rstd, int M, int d,
                                                           float* __restrict__ part) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d) return;
  const int m0 = blockIdx.y * 256, m1 = min(M, m0 + 256);
  float s = 0.f;
  for (int m = m0; m < m1; ++m) s = fmaf(dxn[(size_t)m * d + i] * h[(size_t)m * d + i], rstd[m], s);
  part[(size_t)blockIdx.y * d + i] = s;
}
// column sums of x[M, N] over blocks of 256 rows (bias gradients); k_gain_grad_finish adds the blocks up in order
__global__ void __launch_bounds__(256) k_colsum_partial(const float* __restrict__ x, int M, int N, float* __restrict__ part) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= N) return;
  const int m0 = blockIdx.y * 256, m1 = min(M, m0 + 256);
  float s = 0.f;
  for (int m = m0; m < m1; ++m) s += x[(size_t)m * N + i];
  part[(size_t)blockIdx.y * N + i] = s;
}
__global__ void __launch_bounds__(256) k_gain_grad_finish(const float* __restrict__ part, int n_part, int d,
                                                          float* __restrict__ dgain) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d) return;
  float s = 0.f;
  for (int p = 0; p < n_part; ++p) s += part[(size_t)p * d + i];
  dgain[i] += s;   // the gradient buffer starts at zero; micro-batches add up
}

// dgu from dact: d gate = dact * up * sig(g) (1 + g (1 - sig(g))), d up = dact * silu(g)
__global__ void k_swiglu_bwd(const float* __restrict__ dact, const float* __restrict__ gu, float* __restrict__ dgu, int F,
                             size_t total) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const size_t m = idx / F;
  const int f = (int)(idx % F);
  const float g = gu[m * 2 * F + f], u = gu[m * 2 * F + F + f], da = dact[idx];
  const float sg = 1.0f / (1.0f + expf(-g));
  dgu[m * 2 * F + f] = da * u * sg * (1.0f + g * (1.0f - sg));
  dgu[m * 2 * F + F + f] = da * g * sg;
}

// ---------------------------------------------------------------------------------------
// Fused causal attention in fp32 on the matrix cores (v_mfma_f32_16x16x4_f32), for head dims 16, 32, 64, 128.
// A wave owns 16 positions of one (sequence, head) and walks the other side in tiles of 16; nothing of size
// T x T is stored.  Layouts of one 16x16x4 MFMA: A[m = lane % 16][k = lane / 16], B[k = lane / 16][n = lane % 16],
// D rows 4 (lane / 16) + v (v = 0..3), column lane % 16.  Two kinds of products:
//  * rows x rows over the head dim (scores, dP): both operands are read as float4 per lane - lane (r, g) takes
//    dims 16 w + 4 g + c of row r - and MFMA (w, c) contracts the dims {16 w + 4 g + c : g}: any assignment of dims
//    to k slots is fine as long as both operands use the same one;
//  * (head dim x positions) products over the 16 positions of the tile (P V, dS K, ...): the B operand of MFMA u
//    is the lane's own accumulator entry u of the tile just computed (position 4 g + u), the A operand is the
//    matching row of V / K / Q / dO, read as scalars (lanes along the head dim).
// qkv[M, q + 2 kv] holds rotated q, k and v; out[M, q]; lse[(s Hq + h) T + i].
// ---------------------------------------------------------------------------------------
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int HD>
__device__ __forceinline__ void load_rows4(const float* __restrict__ base, size_t row_stride, int row, int g, float4 (&dst)[HD / 16]) {
#pragma unroll
  for (int w = 0; w < HD / 16; ++w) dst[w] = *(const float4*)(base + (size_t)row * row_stride + 16 * w + 4 * g);
}
__device__ __forceinline__ float f4c(const float4& v, int c) { return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w; }

// acc (rows = positions of `a`, 4 g + v; column = position of `b`, lane % 16) += a b^T over the head dim
template <int HD>
__device__ __forceinline__ f32x4_t dot_rows(const float4 (&a)[HD / 16], const float4 (&b)[HD / 16]) {
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < HD / 16; ++w)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(f4c(a[w], c), f4c(b[w], c), acc, 0, 0, 0);
  return acc;
}
// o (head dims x the 16 columns of lane % 16) += sum over the tile's positions 4 g + u of src[position][dim] * p[u];
// src rows start at `tile_base` (pointer to position 0 of the tile, this head's dims).  Which head dim an
// accumulator entry holds is free to choose (the rows of an MFMA are whatever its A operand's lanes supply):
//   head dims in multiples of 64: lane r supplies the dims 64 j + 4 r + c of a position as float4 loads, so
//     o[4 j + c][v] is dim 64 j + 16 g + 4 v + c;
//   otherwise lane r supplies dim 16 dt + r as scalars: o[dt][v] is dim 16 dt + 4 g + v.
// store_acc writes either arrangement out as float4 runs.
template <int HD>
__device__ __forceinline__ void accumulate_tile(const float* __restrict__ tile_base, size_t row_stride, int n_valid, int g, int r,
                                                const f32x4_t& p, f32x4_t (&o)[HD / 16]) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int pos = min(4 * g + u, n_valid - 1);   // rows past the end repeat the last one (their p is zero)
    const float* row = tile_base + (size_t)pos * row_stride;
    if constexpr (HD % 64 == 0) {
#pragma unroll
      for (int j = 0; j < HD / 64; ++j) {
        const float4 a = *(const float4*)(row + 64 * j + 4 * r);
#pragma unroll
        for (int c = 0; c < 4; ++c) o[4 * j + c] = __builtin_amdgcn_mfma_f32_16x16x4f32(f4c(a, c), p[u], o[4 * j + c], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int dt = 0; dt < HD / 16; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_16x16x4f32(row[16 * dt + r], p[u], o[dt], 0, 0, 0);
    }
  }
}
template <int HD>
__device__ __forceinline__ void store_acc(float* __restrict__ row, const f32x4_t (&o)[HD / 16], int g, float mul) {
  if constexpr (HD % 64 == 0) {
#pragma unroll
    for (int j = 0; j < HD / 64; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        *(float4*)(row + 64 * j + 16 * g + 4 * v) =
            make_float4(o[4 * j][v] * mul, o[4 * j + 1][v] * mul, o[4 * j + 2][v] * mul, o[4 * j + 3][v] * mul);
  } else {
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt)
      *(float4*)(row + 16 * dt + 4 * g) = make_float4(o[dt][0] * mul, o[dt][1] * mul, o[dt][2] * mul, o[dt][3] * mul);
  }
}

template <int HD>
__global__ void __launch_bounds__(256, HD == 128 ? 3 : 1) k_tattn_fwd(const float* __restrict__ qkv, int T, int hq, int hkv, float scale,
                                                   float* __restrict__ out, float* __restrict__ lse) {
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int h = blockIdx.y, s = blockIdx.z, kvh = h / (hq / hkv);
  const int q0 = (blockIdx.x * 4 + wave) * 16;
  if (q0 >= T) return;
  const int qd = hq * HD, kvd = hkv * HD;
  const size_t rl = (size_t)qd + 2 * kvd;
  const float* base = qkv + (size_t)s * T * rl;
  const float* qb = base + (size_t)h * HD;
  const float* kb = base + qd + (size_t)kvh * HD;
  const float* vb = kb + kvd;
  const int qi = min(q0 + r, T - 1);   // this lane's query (columns past T repeat the last one and are not stored)
  float4 qf[HD / 16];
  load_rows4<HD>(qb, rl, qi, g, qf);
  f32x4_t o[HD / 16];
#pragma unroll
  for (int dt = 0; dt < HD / 16; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  const int last = min(q0 + 15, T - 1);
  for (int k0 = 0; k0 <= last; k0 += 16) {
    const int n_valid = min(16, T - k0);
    float4 kf[HD / 16];
    load_rows4<HD>(kb, rl, min(k0 + r, T - 1), g, kf);
    f32x4_t sc = dot_rows<HD>(kf, qf);   // rows: keys k0 + 4 g + v; column: query qi
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int key = k0 + 4 * g + v;
      sc[v] = (key <= qi && key < T) ? sc[v] * scale : -INFINITY;
      mx = fmaxf(mx, sc[v]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);        // finite: key 0 is visible to every query
    const float alpha = expf(m_run - m_new);
    f32x4_t p;
    float ps = 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) { p[v] = expf(sc[v] - m_new); ps += p[v]; }
    l_run = l_run * alpha + ps;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt)
#pragma unroll
      for (int v = 0; v < 4; ++v) o[dt][v] *= alpha;
    accumulate_tile<HD>(vb + (size_t)k0 * rl, rl, n_valid, g, r, p, o);
  }
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (q0 + r >= T) return;
  const float inv = 1.0f / l_run;
  store_acc<HD>(out + ((size_t)s * T + qi) * qd + (size_t)h * HD, o, g, inv);
  if (g == 0) lse[((size_t)s * hq + h) * T + qi] = m_run + logf(l_run);
}

// Backward, queries: a wave owns 16 queries of one (sequence, head).  delta = dO . O; per key tile
//   p = exp(scale s - lse), dP = V dO^T, dS = scale p (dP - delta), dQ^T += K^T dS.
// Writes dq into dqkv's query columns and delta[(s Hq + h) T + i].
template <int HD>
__global__ void __launch_bounds__(256, HD == 128 ? 3 : 1) k_tattn_bwd_q(const float* __restrict__ qkv, const float* __restrict__ out,
                                                     const float* __restrict__ dout, const float* __restrict__ lse, int T, int hq,
                                                     int hkv, float scale, float* __restrict__ dqkv, float* __restrict__ delta) {
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int h = blockIdx.y, s = blockIdx.z, kvh = h / (hq / hkv);
  const int q0 = (blockIdx.x * 4 + wave) * 16;
  if (q0 >= T) return;
  const int qd = hq * HD, kvd = hkv * HD;
  const size_t rl = (size_t)qd + 2 * kvd;
  const float* base = qkv + (size_t)s * T * rl;
  const float* qb = base + (size_t)h * HD;
  const float* kb = base + qd + (size_t)kvh * HD;
  const float* vb = kb + kvd;
  const int qi = min(q0 + r, T - 1);
  float4 qf[HD / 16], dof[HD / 16], of[HD / 16];
  load_rows4<HD>(qb, rl, qi, g, qf);
  load_rows4<HD>(dout + (size_t)s * T * qd + (size_t)h * HD, qd, qi, g, dof);
  load_rows4<HD>(out + (size_t)s * T * qd + (size_t)h * HD, qd, qi, g, of);
  float dl = 0.f;
#pragma unroll
  for (int w = 0; w < HD / 16; ++w)
    dl += dof[w].x * of[w].x + dof[w].y * of[w].y + dof[w].z * of[w].z + dof[w].w * of[w].w;
  dl += __shfl_xor(dl, 16, 64);
  dl += __shfl_xor(dl, 32, 64);
  const size_t stat = ((size_t)s * hq + h) * T + qi;
  const float l = lse[stat];
  f32x4_t dq[HD / 16];
#pragma unroll
  for (int dt = 0; dt < HD / 16; ++dt) dq[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const int last = min(q0 + 15, T - 1);
  for (int k0 = 0; k0 <= last; k0 += 16) {
    const int n_valid = min(16, T - k0);
    float4 kf[HD / 16], vf[HD / 16];
    load_rows4<HD>(kb, rl, min(k0 + r, T - 1), g, kf);
    load_rows4<HD>(vb, rl, min(k0 + r, T - 1), g, vf);
    const f32x4_t sc = dot_rows<HD>(kf, qf);    // rows: keys k0 + 4 g + v; column: query qi
    const f32x4_t dp = dot_rows<HD>(vf, dof);   // dP[key][query] = v_key . dO_query
    f32x4_t ds;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int key = k0 + 4 * g + v;
      const float pv = (key <= qi && key < T) ? expf(sc[v] * scale - l) : 0.f;
      ds[v] = scale * pv * (dp[v] - dl);
    }
    accumulate_tile<HD>(kb + (size_t)k0 * rl, rl, n_valid, g, r, ds, dq);
  }
  if (q0 + r >= T) return;
  store_acc<HD>(dqkv + ((size_t)s * T + qi) * rl + (size_t)h * HD, dq, g, 1.0f);
  if (g == 0) delta[stat] = dl;
}

// Backward, keys and values: a wave owns 16 keys of one (sequence, KV head) and walks the query heads of the
// group and the query tiles from its own on, in that fixed order:
//   p = exp(scale s - lse_q), dV^T += dO^T p, dP = dO V^T, dS = scale p (dP - delta_q), dK^T += Q^T dS.
template <int HD>
__global__ void __launch_bounds__(256, HD == 64 ? 4 : 1) k_tattn_bwd_kv(const float* __restrict__ qkv, const float* __restrict__ dout,
                                                      const float* __restrict__ lse, const float* __restrict__ delta, int T, int hq,
                                                      int hkv, float scale, float* __restrict__ dqkv) {
  const int wave = wave_index(threadIdx.x), lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int kvh = blockIdx.y, s = blockIdx.z, rep = hq / hkv;
  const int k0 = (blockIdx.x * 4 + wave) * 16;
  if (k0 >= T) return;
  const int qd = hq * HD, kvd = hkv * HD;
  const size_t rl = (size_t)qd + 2 * kvd;
  const float* base = qkv + (size_t)s * T * rl;
  const float* kb = base + qd + (size_t)kvh * HD;
  const float* vb = kb + kvd;
  const int kj = min(k0 + r, T - 1);
  const bool key_ok = k0 + r < T;
  float4 kf[HD / 16], vf[HD / 16];
  load_rows4<HD>(kb, rl, kj, g, kf);
  load_rows4<HD>(vb, rl, kj, g, vf);
  f32x4_t dk[HD / 16], dv[HD / 16];
#pragma unroll
  for (int dt = 0; dt < HD / 16; ++dt) { dk[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f}; dv[dt] = dk[dt]; }
  for (int hh = 0; hh < rep; ++hh) {
    const int h = kvh * rep + hh;
    const float* qb = base + (size_t)h * HD;
    const float* dob = dout + (size_t)s * T * qd + (size_t)h * HD;
    const float* lse_h = lse + ((size_t)s * hq + h) * T;
    const float* del_h = delta + ((size_t)s * hq + h) * T;
    for (int q0 = k0; q0 < T; q0 += 16) {
      const int n_valid = min(16, T - q0);
      float4 qf[HD / 16], dof[HD / 16];
      load_rows4<HD>(qb, rl, min(q0 + r, T - 1), g, qf);
      load_rows4<HD>(dob, qd, min(q0 + r, T - 1), g, dof);
      const f32x4_t sc = dot_rows<HD>(qf, kf);    // rows: queries q0 + 4 g + v; column: key kj
      const f32x4_t dp = dot_rows<HD>(dof, vf);   // dP[query][key]
      f32x4_t pv, ds;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int qi = q0 + 4 * g + v;
        const int qc = min(qi, T - 1);
        const float pr = (key_ok && qi < T && kj <= qi) ? expf(sc[v] * scale - lse_h[qc]) : 0.f;
        pv[v] = pr;
        ds[v] = scale * pr * (dp[v] - del_h[qc]);
      }
      accumulate_tile<HD>(dob + (size_t)q0 * qd, qd, n_valid, g, r, pv, dv);
      accumulate_tile<HD>(qb + (size_t)q0 * rl, rl, n_valid, g, r, ds, dk);
    }
  }
  if (!key_ok) return;
  float* krow = dqkv + ((size_t)s * T + kj) * rl + qd + (size_t)kvh * HD;
  store_acc<HD>(krow, dk, g, 1.0f);
  store_acc<HD>(krow + kvd, dv, g, 1.0f);
}

template <int HD>
hipError_t tattn_bwd(const float* qkv, const float* out, const float* dout, const float* lse, int S, int T, int hq, int hkv,
                     float scale, float* dqkv, float* delta, hipStream_t st) {
  const unsigned tiles = (unsigned)((T + 63) / 64);
  hipError_t e = launch(KID_ATTN_GENERIC, k_tattn_bwd_q<HD>, dim3(tiles, hq, S), dim3(256), 0, st, qkv, out, dout, lse, T, hq, hkv,
                        scale, dqkv, delta);
  if (e != hipSuccess) return e;
  return launch(KID_ATTN_GENERIC, k_tattn_bwd_kv<HD>, dim3(tiles, hkv, S), dim3(256), 0, st, qkv, dout, lse, (const float*)delta, T,
                hq, hkv, scale, dqkv);
}

// Attention backward pieces (the contractions are batched GEMMs):
// delta[(s Hq + h) T + i] = dO_i . O_i over the head's dims; one wave per (s, i, h)
__global__ void __launch_bounds__(64) k_attn_delta(const float* __restrict__ dout, const float* __restrict__ out, int T, int hq,
                                                   int hd, float* __restrict__ delta) {
  const size_t b = blockIdx.x;            // (s * T + i) * hq + h
  const int h = (int)(b % hq);
  const size_t si = b / hq, s = si / T, i = si % T;
  const float* a = dout + (si * hq + h) * hd;
  const float* o = out + (si * hq + h) * hd;
  float d = 0.f;
  for (int e = threadIdx.x; e < hd; e += 64) d = fmaf(a[e], o[e], d);
  d = wave_reduce_sum(d);
  if (threadIdx.x == 0) delta[(s * hq + h) * T + i] = d;
}
// d(q . k)_ij = scale * p_ij (dP_ij - delta_i), in place over dP
__global__ void k_dscores(const float* __restrict__ prob, float* __restrict__ dp, const float* __restrict__ delta, int T,
                          float scale, size_t total) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const float pr = prob[idx];   // zero above the diagonal, where dP was not computed
  dp[idx] = pr == 0.f ? 0.f : scale * pr * (dp[idx] - delta[idx / T]);
}

// Embedding rows: dE[tokens[m]] += dh[m].  Workgroup b owns the token ids congruent to b modulo the grid size
// and walks the rows in order m = 0, 1, ..., 256 at a time: one id, one owner, one order of additions.
__global__ void __launch_bounds__(256) k_embed_bwd(const int32_t* __restrict__ tokens, const float* __restrict__ dh, int M, int d,
                                                   int V, float* __restrict__ dE) {
  __shared__ int s_tok[256];
  for (int m0 = 0; m0 < M; m0 += 256) {
    const int m = m0 + threadIdx.x;
    int tok = -1;
    if (m < M) {
      tok = clamp_token(tokens[m], V);
      if (tok % (int)gridDim.x != (int)blockIdx.x) tok = -1;
    }
    __syncthreads();   // the previous round's list has been read
    s_tok[threadIdx.x] = tok;
    __syncthreads();
    for (int j = 0; j < 256; ++j) {
      const int t = s_tok[j];   // the same for every thread
      if (t < 0) continue;
      const float* src = dh + (size_t)(m0 + j) * d;
      float* dst = dE + (size_t)t * d;
      for (int i = threadIdx.x; i < d; i += 256) dst[i] += src[i];
    }
  }
}

// Adam (Kingma & Ba, Algorithm 1): c1 = 1 - beta1^t, c2 = 1 - beta2^t
__global__ void k_adam(float* __restrict__ theta, const float* __restrict__ g, float* __restrict__ m, float* __restrict__ v,
                       size_t n, float lr, float beta1, float beta2, float eps, float c1, float c2) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float gi = g[i];
  const float mi = beta1 * m[i] + (1.0f - beta1) * gi;
  const float vi = beta2 * v[i] + (1.0f - beta2) * gi * gi;
  m[i] = mi;
  v[i] = vi;
  theta[i] -= lr * (mi / c1) / (sqrtf(vi / c2) + eps);
}

unsigned blocks256(size_t n) { return (unsigned)((n + 255) / 256); }

}  // namespace

// ---------------------------------------------------------------------------------------
// the trainer
// ---------------------------------------------------------------------------------------
struct sapo_trainer {
  sapo_model_config cfg;
  sapo_adam_config opt;
  int t = 0;                      // Adam steps taken
  int pieces = 3;                 // bf16 pieces per value in the large GEMMs: 3 (fp32 accuracy), 2 or 1 (bf16 operands)
  bool use_bias = false;          // the model has biases on its query / key / value projections (set_qkv_bias)
  int n_in = 0;                   // tensors of the input list; tensor n_in + l is layer l's bias vector
  int device = 0;
  size_t n_params = 0;
  float* theta = nullptr;         // [n_params] masters, tensors back to back in tensor-list order
  float* grad = nullptr;
  float* m = nullptr;
  float* v = nullptr;
  float2* rope = nullptr;         // [max_seq][hd / 2] (cos, sin)
  std::vector<size_t> off, len;   // per tensor
};

namespace {

struct Dims {
  size_t d, q, kv, nqkv, F, V;
  int L;
  explicit Dims(const sapo_model_config& c)
      : d(c.d_model), q((size_t)c.n_q_heads * c.head_dim), kv((size_t)c.n_kv_heads * c.head_dim), nqkv(q + 2 * kv), F(c.d_ff),
        V(c.vocab), L(c.n_layers) {}
};

int n_tensors_of(const sapo_model_config& c) { return 1 + 9 * c.n_layers + 1 + (c.tied_embeddings ? 0 : 1); }

void tensor_sizes(const sapo_model_config& c, std::vector<size_t>& len) {
  const Dims D(c);
  len.clear();
  len.push_back(D.V * D.d);
  for (int l = 0; l < D.L; ++l) {
    const size_t s[9] = {D.d, D.q * D.d, D.kv * D.d, D.kv * D.d, D.d * D.q, D.d, D.F * D.d, D.F * D.d, D.d * D.F};
    for (size_t x : s) len.push_back(x);
  }
  len.push_back(D.d);
  if (!c.tied_embeddings) len.push_back(D.V * D.d);
  for (int l = 0; l < D.L; ++l) len.push_back(D.nqkv);   // optional projection biases [bq | bk | bv] (zero and idle unless set)
}

// rows of logits held at once: about 2.5 GB (enough rows for the d-input GEMM of the head, whose output is only
// d_model wide, to fill the chip), a multiple of the GEMM tile
size_t lm_chunk_rows(const Dims& D, size_t M) {
  size_t r = ((size_t)5 << 29) / (D.V * sizeof(float)) / 128 * 128;
  if (r < 128) r = 128;
  return r < M ? r : M;
}

struct Arena {
  char* base;
  size_t off;
  template <typename T> T* take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

// GEMMs with a long contraction whose output tiles do not fill the resident workgroups (the weight gradients; the
// head's d-input product: 238 tiles, contraction over the vocabulary) are split over the contraction into up to
// kMaxSplits parts that are added in part order; the buffer holds 8 parts of the largest layer matrix.
inline size_t split_parts_floats(const Dims& D) { return (size_t)8 * std::max((size_t)2 * D.F * D.d, (size_t)192 * 128 * 128); }
constexpr int kPieces = 3;   // most bf16 pieces per fp32 value in the packed GEMMs (3: fp32 accuracy; buffers are sized for it)

// the fused attention kernels need float4 rows: head dim 16 / 32 / 64 / 128 and row lengths that are multiples of 4
inline bool fused_attention(const sapo_model_config& c) {
  const int hd = c.head_dim;
  return (hd == 16 || hd == 32 || hd == 64 || hd == 128) && (c.n_q_heads * hd) % 4 == 0 && (c.n_kv_heads * hd) % 4 == 0;
}

struct LayerActs {
  float *h, *r1, *xn, *qkv, *lse, *ao, *h2, *r2, *xn2, *gu, *act;
};
struct TrainPlan {
  std::vector<LayerActs> layer;
  float *h_last, *rf, *xf;                      // final residual rows, their rstd, final-normed rows
  float* xfc;                                   // the final-normed rows that predict a masked token, gathered
  int *mrows, *mpos, *mcount;                   // per micro-batch: those rows' indices (mpos: their (s, t)), their number
  float *dh, *dx, *dact, *dgu, *dao, *dqkv;     // backward temporaries
  float *delta, *prob, *dsc, *gpart, *logits, *logp_all, *loss;
  void* sur_ws;
  long long* n_masked;
  float* kparts;                                // partial products of the split weight-gradient GEMMs
  char *packa, *packb, *head_nt, *head_t;       // packed operands; the LM head packed once per update, both ways
  size_t packa_cap, packb_cap, head_cap, head_t_cap;
  size_t chunk;
  size_t bytes;
};

void make_plan(const sapo_model_config& c, size_t S, size_t T, size_t S_total, char* base, TrainPlan& p) {
  const Dims D(c);
  const size_t M = S * T;
  Arena A{base, 0};
  p.layer.resize(D.L);
  for (int l = 0; l < D.L; ++l) {
    LayerActs& a = p.layer[l];
    a.h = A.take<float>(M * D.d);
    a.r1 = A.take<float>(M);
    a.xn = A.take<float>(M * D.d);
    a.qkv = A.take<float>(M * D.nqkv);
    a.lse = A.take<float>(S * c.n_q_heads * T);
    a.ao = A.take<float>(M * D.q);
    a.h2 = A.take<float>(M * D.d);
    a.r2 = A.take<float>(M);
    a.xn2 = A.take<float>(M * D.d);
    a.gu = A.take<float>(M * 2 * D.F);
    a.act = A.take<float>(M * D.F);
  }
  p.h_last = A.take<float>(M * D.d);
  p.rf = A.take<float>(M);
  p.xf = A.take<float>(M * D.d);
  p.xfc = A.take<float>(M * D.d);
  p.mrows = A.take<int>(S_total * T);
  p.mpos = A.take<int>(2 * M);
  p.mcount = A.take<int>((S_total + S - 1) / S);
  p.dh = A.take<float>(M * D.d);
  p.dx = A.take<float>(M * D.d);
  p.dact = A.take<float>(M * D.F);
  p.dgu = A.take<float>(M * 2 * D.F);
  p.dao = A.take<float>(M * D.q);
  p.dqkv = A.take<float>(M * D.nqkv);
  p.delta = A.take<float>(S * c.n_q_heads * T);
  // T x T score matrices: only for head dims the fused attention kernels do not take
  const size_t n_tt = fused_attention(c) ? 0 : S * c.n_q_heads * T * T;
  p.prob = A.take<float>(n_tt);
  p.dsc = A.take<float>(n_tt);
  p.gpart = A.take<float>(((M + 255) / 256) * std::max(D.d, D.nqkv));
  p.chunk = lm_chunk_rows(D, M);
  p.logits = A.take<float>(p.chunk * D.V);
  p.logp_all = A.take<float>(S_total * T);   // log-probs of the whole training set (micro-batches fill their rows)
  p.loss = A.take<float>(4);
  p.n_masked = A.take<long long>(1);
  p.kparts = A.take<float>(split_parts_floats(D));
  // packed GEMM operands: the largest row-side (A) and column-side (B) operand of any GEMM of the update
  {
    const size_t R = p.chunk, twoF = 2 * D.F;
    const size_t a_shapes[][2] = {{M, D.d}, {M, D.q}, {M, D.F}, {M, twoF}, {M, D.nqkv}, {D.d, M}, {twoF, M}, {D.nqkv, M},
                                  {R, D.d}, {R, D.V}, {D.V, R}};
    const size_t b_shapes[][2] = {{D.nqkv, D.d}, {D.d, D.q}, {twoF, D.d}, {D.d, D.F}, {D.F, D.d}, {D.F, M}, {D.d, twoF},
                                  {D.d, M}, {D.q, D.d}, {D.q, M}, {D.d, D.nqkv}, {D.d, R}};
    p.packa_cap = p.packb_cap = 0;
    for (auto& sh : a_shapes) p.packa_cap = std::max(p.packa_cap, x3_pack_bytes(kPieces, sh[0], sh[1]));
    for (auto& sh : b_shapes) p.packb_cap = std::max(p.packb_cap, x3_pack_bytes(kPieces, sh[0], sh[1]));
    p.head_cap = x3_pack_bytes(kPieces, D.V, D.d);
    p.head_t_cap = x3_pack_bytes(kPieces, D.d, D.V);
    p.packa = A.take<char>(p.packa_cap);
    p.packb = A.take<char>(p.packb_cap);
    p.head_nt = A.take<char>(p.head_cap);
    p.head_t = A.take<char>(p.head_t_cap);
  }
  p.sur_ws = A.take<char>(g_surrogate_workspace_bytes());
  p.bytes = (A.off + 255) & ~(size_t)255;
}

int check_cfg(const sapo_model_config* c) {
  if (!c) return set_error(SAPO_EINVAL, "cfg is NULL");
  if (c->n_layers <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->d_ff <= 0 ||
      c->vocab <= 0 || c->max_seq <= 0)
    return set_error(SAPO_EINVAL, "model sizes must be positive");
  if (c->n_q_heads % c->n_kv_heads != 0) return set_error(SAPO_ESHAPE, "n_q_heads must be a multiple of n_kv_heads");
  if (c->head_dim % 2 != 0 || c->head_dim > 128) return set_error(SAPO_ESHAPE, "head_dim must be even and at most 128");
  if (c->dtype != SAPO_DTYPE_F32 && c->dtype != SAPO_DTYPE_BF16) return set_error(SAPO_EINVAL, "unknown dtype");
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) return set_error(SAPO_EINVAL, "rms_eps and rope_theta must be > 0");
  return SAPO_OK;
}

bool gain_tensor(const sapo_model_config& c, int i) {
  if (i == 0) return false;
  const int last_layer_tensor = 9 * c.n_layers;
  if (i <= last_layer_tensor) { const int k = (i - 1) % 9; return k == 0 || k == 5; }
  return i == last_layer_tensor + 1;
}

}  // namespace

extern "C" void sapo_trainer_destroy(sapo_trainer* tr) {
  if (!tr) return;
  (void)hipSetDevice(tr->device);
  for (void* p : {(void*)tr->theta, (void*)tr->grad, (void*)tr->m, (void*)tr->v, (void*)tr->rope})
    if (p) (void)hipFree(p);
  delete tr;
}

extern "C" int sapo_trainer_create(const sapo_model_config* cfg, const void* const* tensors, int n_tensors,
                                   const sapo_adam_config* opt, void* stream, sapo_trainer** out) {
  if (!out) return set_error(SAPO_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (!tensors) return set_error(SAPO_EINVAL, "tensors is NULL");
  if (n_tensors != n_tensors_of(*cfg))
    return set_error(SAPO_EINVAL, "n_tensors is %d, expected %d", n_tensors, n_tensors_of(*cfg));
  for (int i = 0; i < n_tensors; ++i)
    if (!tensors[i]) return set_error(SAPO_EINVAL, "tensor %d is NULL", i);
  sapo_adam_config o{1e-3f, 0.9f, 0.999f, 1e-8f};
  if (opt) o = *opt;
  if (!(o.lr > 0.f) || !(o.beta1 >= 0.f && o.beta1 < 1.f) || !(o.beta2 >= 0.f && o.beta2 < 1.f) || !(o.eps > 0.f))
    return set_error(SAPO_EINVAL, "Adam needs lr > 0, beta1 and beta2 in [0, 1), eps > 0");
  hipStream_t st = (hipStream_t)stream;
  sapo_trainer* tr = new sapo_trainer;
  tr->cfg = *cfg;
  tr->opt = o;
  (void)hipGetDevice(&tr->device);
  tensor_sizes(*cfg, tr->len);
  tr->off.resize(tr->len.size());
  size_t n = 0;
  for (size_t i = 0; i < tr->len.size(); ++i) { tr->off[i] = n; n += tr->len[i]; }
  tr->n_params = n;
  tr->n_in = n_tensors;
  auto bail = [&](int code) { sapo_trainer_destroy(tr); return code; };
  for (float** p : {&tr->theta, &tr->grad, &tr->m, &tr->v}) {
    hipError_t e = hipMalloc((void**)p, n * sizeof(float));
    if (e != hipSuccess) return bail(set_error(SAPO_EHIP, "hipMalloc of %zu bytes failed: %s", n * sizeof(float), hipGetErrorString(e)));
  }
  for (int i = 0; i < n_tensors; ++i) {
    float* dst = tr->theta + tr->off[i];
    hipError_t e;
    if (cfg->dtype == SAPO_DTYPE_F32 || gain_tensor(*cfg, i))
      e = hipMemcpyAsync(dst, tensors[i], tr->len[i] * sizeof(float), hipMemcpyDeviceToDevice, st);
    else
      e = launch(KID_MISC, k_bf16_to_f32, dim3(blocks256(tr->len[i])), dim3(256), 0, st, (const bf16*)tensors[i], dst, tr->len[i]);
    if (e != hipSuccess) return bail(set_error(SAPO_EHIP, "copy of tensor %d failed: %s", i, hipGetErrorString(e)));
  }
  for (float* p : {tr->grad, tr->m, tr->v}) {
    hipError_t e = g_fill_f32(p, 0.f, n, st);
    if (e != hipSuccess) return bail(set_error(SAPO_EHIP, "fill failed: %s", hipGetErrorString(e)));
  }
  {
    const size_t b0 = tr->off[n_tensors];   // the bias vectors start at zero
    hipError_t e = g_fill_f32(tr->theta + b0, 0.f, n - b0, st);
    if (e != hipSuccess) return bail(set_error(SAPO_EHIP, "fill failed: %s", hipGetErrorString(e)));
  }
  const int half = cfg->head_dim / 2;
  std::vector<float2> tab((size_t)cfg->max_seq * half);
  for (int pos = 0; pos < cfg->max_seq; ++pos)
    for (int i = 0; i < half; ++i) {
      const double ang = (double)pos * pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
      tab[(size_t)pos * half + i] = make_float2((float)cos(ang), (float)sin(ang));
    }
  hipError_t e = hipMalloc((void**)&tr->rope, tab.size() * sizeof(float2));
  if (e == hipSuccess) e = hipMemcpy(tr->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
  if (e != hipSuccess) return bail(set_error(SAPO_EHIP, "rotary table: %s", hipGetErrorString(e)));
  *out = tr;
  return SAPO_OK;
}

extern "C" size_t sapo_trainer_workspace_bytes(const sapo_trainer* tr, int S, int T) {
  if (!tr || S <= 0 || T < 2 || T > tr->cfg.max_seq) return 0;
  TrainPlan p;
  make_plan(tr->cfg, (size_t)S, (size_t)T, (size_t)S, nullptr, p);
  return p.bytes;
}

extern "C" size_t sapo_trainer_workspace_bytes_for(const sapo_trainer* tr, int S, int T, int S_micro) {
  if (!tr || S <= 0 || T < 2 || T > tr->cfg.max_seq || S_micro <= 0 || S_micro > S) return 0;
  TrainPlan p;
  make_plan(tr->cfg, (size_t)S_micro, (size_t)T, (size_t)S, nullptr, p);
  return p.bytes;
}

extern "C" int sapo_trainer_set_qkv_bias(sapo_trainer* tr, int layer, const float* bq, const float* bk, const float* bv,
                                         void* stream) {
  if (!tr || !bq || !bk || !bv) return set_error(SAPO_EINVAL, "NULL argument");
  if (layer < 0 || layer >= tr->cfg.n_layers) return set_error(SAPO_EINVAL, "layer %d out of range", layer);
  const Dims D(tr->cfg);
  float* dst = tr->theta + tr->off[tr->n_in + layer];
  hipStream_t st = (hipStream_t)stream;
  T_CK(hipMemcpyAsync(dst, bq, D.q * sizeof(float), hipMemcpyDeviceToDevice, st));
  T_CK(hipMemcpyAsync(dst + D.q, bk, D.kv * sizeof(float), hipMemcpyDeviceToDevice, st));
  T_CK(hipMemcpyAsync(dst + D.q + D.kv, bv, D.kv * sizeof(float), hipMemcpyDeviceToDevice, st));
  tr->use_bias = true;
  return SAPO_OK;
}

extern "C" int sapo_trainer_get_qkv_bias(const sapo_trainer* tr, int layer, float* bq, float* bk, float* bv, void* stream) {
  if (!tr || !bq || !bk || !bv) return set_error(SAPO_EINVAL, "NULL argument");
  if (layer < 0 || layer >= tr->cfg.n_layers) return set_error(SAPO_EINVAL, "layer %d out of range", layer);
  const Dims D(tr->cfg);
  const float* src = tr->theta + tr->off[tr->n_in + layer];
  hipStream_t st = (hipStream_t)stream;
  T_CK(hipMemcpyAsync(bq, src, D.q * sizeof(float), hipMemcpyDeviceToDevice, st));
  T_CK(hipMemcpyAsync(bk, src + D.q, D.kv * sizeof(float), hipMemcpyDeviceToDevice, st));
  T_CK(hipMemcpyAsync(bv, src + D.q + D.kv, D.kv * sizeof(float), hipMemcpyDeviceToDevice, st));
  return SAPO_OK;
}

extern "C" int sapo_trainer_steps(const sapo_trainer* tr) { return tr ? tr->t : -1; }

extern "C" int sapo_trainer_set_matmul_pieces(sapo_trainer* tr, int pieces) {
  if (!tr) return set_error(SAPO_EINVAL, "trainer is NULL");
  if (pieces < 1 || pieces > 3)
    return set_error(SAPO_EINVAL, "pieces must be 3 (fp32 accuracy), 2 (16 significant bits) or 1 (bf16 operands)");
  tr->pieces = pieces;
  return SAPO_OK;
}

extern "C" int sapo_trainer_read(const sapo_trainer* tr, int what, int tensor, float* out, size_t n, void* stream) {
  if (!tr || !out) return set_error(SAPO_EINVAL, "NULL argument");
  if (tensor < 0 || tensor >= (int)tr->len.size()) return set_error(SAPO_EINVAL, "tensor index %d out of range", tensor);
  if (n != tr->len[tensor]) return set_error(SAPO_EINVAL, "tensor %d has %zu elements, not %zu", tensor, tr->len[tensor], n);
  const float* src = what == 0 ? tr->theta : what == 1 ? tr->grad : what == 2 ? tr->m : what == 3 ? tr->v : nullptr;
  if (!src) return set_error(SAPO_EINVAL, "what must be 0 (parameters), 1 (gradient), 2 or 3 (Adam moments)");
  T_CK(hipMemcpyAsync(out, src + tr->off[tensor], n * sizeof(float), hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return SAPO_OK;
}

extern "C" int sapo_trainer_export(const sapo_trainer* tr, void* const* tensors_out, int n_tensors, void* stream) {
  if (!tr || !tensors_out) return set_error(SAPO_EINVAL, "NULL argument");
  if (n_tensors != tr->n_in) return set_error(SAPO_EINVAL, "n_tensors is %d, expected %d", n_tensors, tr->n_in);
  hipStream_t st = (hipStream_t)stream;
  for (int i = 0; i < n_tensors; ++i) {
    if (!tensors_out[i]) return set_error(SAPO_EINVAL, "tensor %d is NULL", i);
    const float* src = tr->theta + tr->off[i];
    if (tr->cfg.dtype == SAPO_DTYPE_F32 || gain_tensor(tr->cfg, i))
      T_CK(hipMemcpyAsync(tensors_out[i], src, tr->len[i] * sizeof(float), hipMemcpyDeviceToDevice, st));
    else
      T_CK(launch(KID_MISC, k_f32_to_bf16, dim3(blocks256(tr->len[i])), dim3(256), 0, st, src, (bf16*)tensors_out[i], tr->len[i]));
  }
  return SAPO_OK;
}

// Forward, LM head and backward over one micro-batch of S_ sequences: gradients are added to tr->grad, the
// log-probs go to logp_new [S_, T_].  p.n_masked holds the count of masked tokens of the whole training set and
// the LM head is packed (p.head_nt, p.head_t).
static int update_rows(sapo_trainer* tr, const TrainPlan& p, const int32_t* tokens, const uint8_t* completion_mask,
                       const float* logp_old, const float* advantages, int S_, int T_, float eps_low, float eps_high,
                       float* logp_new, const int* rows, int n_rows, hipStream_t st) {
  const sapo_model_config& c = tr->cfg;
  const Dims D(c);
  const size_t S = S_, T = T_, M = S * T;
  const int d = (int)D.d, q = (int)D.q, kv = (int)D.kv, nqkv = (int)D.nqkv, F = (int)D.F, V = (int)D.V;
  const int hq = c.n_q_heads, hkv = c.n_kv_heads, hd = c.head_dim;
  const int Mi = (int)M;
  auto TH = [&](int tensor) { return tr->theta + tr->off[tensor]; };
  auto GR = [&](int tensor) { return tr->grad + tr->off[tensor]; };
  const int t_final = 1 + 9 * D.L, t_head = c.tied_embeddings ? 0 : t_final + 1;
  const int rep = hq / hkv;
  const float att_scale = 1.0f / sqrtf((float)hd);
  const bool fused_attn = fused_attention(c);
  const size_t n_sc = S * hq * T * T;
  const long TT = (long)(T * T), Trow = (long)(T * D.nqkv), Tq = (long)(T * D.q);
  Batch b_scores, b_pv, b_dp, b_dq, b_dk, b_dv;
  // per (sequence, query head): Q_h and the group's K -> scores
  b_scores.nh = hq; b_scores.bdiv = rep; b_scores.count = S_ * hq;
  b_scores.a1 = Trow; b_scores.a2 = hd; b_scores.b1 = Trow; b_scores.b2 = hd; b_scores.c1 = hq * TT; b_scores.c2 = TT;
  // P and the group's V -> the head's columns of the attention output
  b_pv = b_scores; b_pv.a1 = hq * TT; b_pv.a2 = TT; b_pv.c1 = Tq; b_pv.c2 = hd;
  // dO_h and the group's V -> dP
  b_dp = b_scores; b_dp.a1 = Tq; b_dp.a2 = hd;
  // dS and the group's K -> dQ_h
  b_dq = b_scores; b_dq.a1 = hq * TT; b_dq.a2 = TT; b_dq.c1 = Trow; b_dq.c2 = hd;
  // per (sequence, KV head), one query head of the group at a time: dS_h^T Q_h -> dK, P_h^T dO_h -> dV
  b_dk.nh = hkv; b_dk.bdiv = 1; b_dk.count = S_ * hkv;
  b_dk.a1 = hq * TT; b_dk.a2 = rep * TT; b_dk.b1 = Trow; b_dk.b2 = (long)rep * hd; b_dk.c1 = Trow; b_dk.c2 = hd;
  b_dv = b_dk; b_dv.b1 = Tq;
  b_scores.causal = 1; b_dp.causal = 1; b_pv.causal = 2; b_dq.causal = 2; b_dk.causal = 3; b_dv.causal = 3;

  // The projections and the LM head run on the packed bf16-piece GEMM; forms as in sgemm<TA, TB>.
  const int pieces = tr->pieces;
  const X3Bufs xb{p.packa, p.packb, p.packa_cap, p.packb_cap, pieces, p.kparts, split_parts_floats(D)};
  auto mm_nt = [&](const float* X, int ldx, const float* W, int ldw, float* C, int ldc, int M_, int N_, int K_, float beta,
                   const void* w_packed = nullptr) {   // C = beta C + X W^T
    return gemm_x3(X3Op{X, ldx, M_, K_, false}, X3Op{W, ldw, N_, K_, false}, C, ldc, beta, xb, st, false, nullptr, w_packed);
  };
  auto mm_nn = [&](const float* A_, int lda, const float* B_, int ldb, float* C, int ldc, int M_, int N_, int K_, float beta,
                   const void* b_packed = nullptr) {   // C = beta C + A B
    return gemm_x3(X3Op{A_, lda, M_, K_, false}, X3Op{B_, ldb, N_, K_, true}, C, ldc, beta, xb, st, true, nullptr, b_packed);
  };
  auto mm_tn = [&](const float* A_, int lda, const float* B_, int ldb, float* C, int Mg, int Ng, int Kg, float beta) {
    return gemm_x3(X3Op{A_, lda, Mg, Kg, true}, X3Op{B_, ldb, Ng, Kg, true}, C, Ng, beta, xb, st, true);   // C = beta C + A^T B
  };

  // ---- forward, every activation kept
  float* h = p.layer[0].h;
  T_CK(launch(KID_EMBED, k_embed_rows, dim3(Mi), dim3(256), 0, st, tokens, (const float*)TH(0), h, d, V));
  for (int l = 0; l < D.L; ++l) {
    const LayerActs& a = p.layer[l];
    const int t0 = 1 + 9 * l;   // attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down
    T_CK(launch(KID_RMSNORM, k_rmsnorm_fwd, dim3(Mi), dim3(256), 0, st, (const float*)a.h, (const float*)TH(t0), c.rms_eps, d,
                a.xn, a.r1));
    T_CK(mm_nt(a.xn, d, TH(t0 + 1), d, a.qkv, nqkv, Mi, nqkv, d, 0.f));   // wq, wk, wv are adjacent
    if (tr->use_bias) T_CK(g_add_row_bias(a.qkv, TH(tr->n_in + l), Mi, nqkv, st));
    {
      const size_t total = M * (size_t)(hq + hkv) * (hd / 2);
      T_CK(launch(KID_ROPE_APPEND, k_rope, dim3(blocks256(total)), dim3(256), 0, st, a.qkv, (const float2*)tr->rope, (int)T,
                  hq + hkv, hd, nqkv, 1.0f, total));
    }
    if (fused_attn) {
      const dim3 ag((unsigned)((T + 63) / 64), hq, (unsigned)S);
      hipError_t e = hipErrorInvalidValue;
      if (hd == 16) e = launch(KID_ATTN_GENERIC, k_tattn_fwd<16>, ag, dim3(256), 0, st, (const float*)a.qkv, (int)T, hq, hkv, att_scale, a.ao, a.lse);
      if (hd == 32) e = launch(KID_ATTN_GENERIC, k_tattn_fwd<32>, ag, dim3(256), 0, st, (const float*)a.qkv, (int)T, hq, hkv, att_scale, a.ao, a.lse);
      if (hd == 64) e = launch(KID_ATTN_GENERIC, k_tattn_fwd<64>, ag, dim3(256), 0, st, (const float*)a.qkv, (int)T, hq, hkv, att_scale, a.ao, a.lse);
      if (hd == 128) e = launch(KID_ATTN_GENERIC, k_tattn_fwd<128>, ag, dim3(256), 0, st, (const float*)a.qkv, (int)T, hq, hkv, att_scale, a.ao, a.lse);
      T_CK(e);
    } else {
      T_CK((sgemm<0, 1>(a.qkv, nqkv, a.qkv + q, nqkv, p.prob, (int)T, (int)T, (int)T, hd, 0.f, st, b_scores)));
      T_CK(launch(KID_ATTN_GENERIC, k_softmax_causal, dim3((unsigned)(S * hq * T)), dim3(64), 0, st, p.prob, a.lse, (int)T,
                  att_scale));
      T_CK((sgemm<0, 0>(p.prob, (int)T, a.qkv + q + kv, nqkv, a.ao, q, (int)T, hd, (int)T, 0.f, st, b_pv)));
    }
    T_CK(hipMemcpyAsync(a.h2, a.h, M * D.d * sizeof(float), hipMemcpyDeviceToDevice, st));
    T_CK(mm_nt(a.ao, q, TH(t0 + 4), q, a.h2, d, Mi, d, q, 1.f));
    T_CK(launch(KID_RMSNORM, k_rmsnorm_fwd, dim3(Mi), dim3(256), 0, st, (const float*)a.h2, (const float*)TH(t0 + 5), c.rms_eps,
                d, a.xn2, a.r2));
    T_CK(mm_nt(a.xn2, d, TH(t0 + 6), d, a.gu, 2 * F, Mi, 2 * F, d, 0.f));   // w_gate, w_up are adjacent
    T_CK(launch(KID_SWIGLU, k_swiglu_fwd, dim3(blocks256(M * D.F)), dim3(256), 0, st, (const float*)a.gu, a.act, F, M * D.F));
    float* h_next = (l + 1 < D.L) ? p.layer[l + 1].h : p.h_last;
    T_CK(hipMemcpyAsync(h_next, a.h2, M * D.d * sizeof(float), hipMemcpyDeviceToDevice, st));
    T_CK(mm_nt(a.act, F, TH(t0 + 8), F, h_next, d, Mi, d, F, 1.f));
  }
  T_CK(launch(KID_RMSNORM, k_rmsnorm_fwd, dim3(Mi), dim3(256), 0, st, (const float*)p.h_last, (const float*)TH(t_final),
              c.rms_eps, d, p.xf, p.rf));

  // ---- LM head, over the rows that predict a masked token only (the others have no log-prob to report and a zero
  // d logits row): their final-normed rows gathered, then chunks of them: logits, log-probs, d logits, d rows (into
  // p.dh, scattered to p.dx afterwards) and d head
  T_CK(g_fill_f32(logp_new, 0.f, M, st));
  T_CK(g_fill_f32(p.dx, 0.f, M * D.d, st));
  if (n_rows > 0) {
    T_CK(launch(KID_MISC, k_move_rows, dim3(n_rows), dim3(256), 0, st, (const float*)p.xf, rows, d, 0, p.xfc));
    for (size_t r0 = 0; r0 < (size_t)n_rows; r0 += p.chunk) {
      const int R = (int)(((size_t)n_rows - r0 < p.chunk) ? (size_t)n_rows - r0 : p.chunk);
      T_CK(mm_nt(p.xfc + r0 * D.d, d, TH(t_head), d, p.logits, V, R, V, d, 0.f, p.head_nt));
      T_CK(launch(KID_SCORE_ROWS, k_logp_dlogits, dim3(R), dim3(256), 0, st, p.logits, V, rows + r0, (int)T, tokens, completion_mask,
                  logp_old, advantages, eps_low, eps_high, (const long long*)p.n_masked, logp_new));
      T_CK(mm_nn(p.logits, V, TH(t_head), d, p.dh + r0 * D.d, d, R, d, V, 0.f, p.head_t));
      T_CK(mm_tn(p.logits, V, p.xfc + r0 * D.d, d, GR(t_head), V, d, R, 1.f));
    }
    T_CK(launch(KID_MISC, k_move_rows, dim3(n_rows), dim3(256), 0, st, (const float*)p.dh, rows, d, 1, p.dx));
  }
  // ---- backward through the layers
  const int n_gpart = (Mi + 255) / 256;
  auto norm_bwd = [&](const float* dxn, const float* hin, const float* rstd, int gain_tensor_idx, int accumulate) -> hipError_t {
    hipError_t e = launch(KID_MISC, k_gain_grad_partial, dim3((d + 255) / 256, n_gpart), dim3(256), 0, st, dxn, hin, rstd, Mi, d,
                          p.gpart);
    if (e != hipSuccess) return e;
    e = launch(KID_MISC, k_gain_grad_finish, dim3((d + 255) / 256), dim3(256), 0, st, (const float*)p.gpart, n_gpart, d,
               GR(gain_tensor_idx));
    if (e != hipSuccess) return e;
    return launch(KID_RMSNORM, k_rmsnorm_bwd, dim3(Mi), dim3(256), 0, st, dxn, hin, rstd, (const float*)TH(gain_tensor_idx), d,
                  p.dh, accumulate);
  };
  T_CK(norm_bwd(p.dx, p.h_last, p.rf, t_final, 0));
  for (int l = D.L - 1; l >= 0; --l) {
    const LayerActs& a = p.layer[l];
    const int t0 = 1 + 9 * l;
    // down projection
    T_CK(mm_nn(p.dh, d, TH(t0 + 8), F, p.dact, F, Mi, F, d, 0.f));
    T_CK(mm_tn(p.dh, d, a.act, F, GR(t0 + 8), d, F, Mi, 1.f));
    T_CK(launch(KID_SWIGLU, k_swiglu_bwd, dim3(blocks256(M * D.F)), dim3(256), 0, st, (const float*)p.dact, (const float*)a.gu,
                p.dgu, F, M * D.F));
    // gate / up projections
    T_CK(mm_nn(p.dgu, 2 * F, TH(t0 + 6), d, p.dx, d, Mi, d, 2 * F, 0.f));
    T_CK(mm_tn(p.dgu, 2 * F, a.xn2, d, GR(t0 + 6), 2 * F, d, Mi, 1.f));
    T_CK(norm_bwd(p.dx, a.h2, a.r2, t0 + 5, 1));
    // output projection
    T_CK(mm_nn(p.dh, d, TH(t0 + 4), q, p.dao, q, Mi, q, d, 0.f));
    T_CK(mm_tn(p.dh, d, a.ao, q, GR(t0 + 4), d, q, Mi, 1.f));
    // attention and the rotary embedding
    if (fused_attn) {
      hipError_t e = hipErrorInvalidValue;
      if (hd == 16) e = tattn_bwd<16>(a.qkv, a.ao, p.dao, a.lse, S_, T_, hq, hkv, att_scale, p.dqkv, p.delta, st);
      if (hd == 32) e = tattn_bwd<32>(a.qkv, a.ao, p.dao, a.lse, S_, T_, hq, hkv, att_scale, p.dqkv, p.delta, st);
      if (hd == 64) e = tattn_bwd<64>(a.qkv, a.ao, p.dao, a.lse, S_, T_, hq, hkv, att_scale, p.dqkv, p.delta, st);
      if (hd == 128) e = tattn_bwd<128>(a.qkv, a.ao, p.dao, a.lse, S_, T_, hq, hkv, att_scale, p.dqkv, p.delta, st);
      T_CK(e);
    } else {
      T_CK((sgemm<0, 1>(a.qkv, nqkv, a.qkv + q, nqkv, p.prob, (int)T, (int)T, (int)T, hd, 0.f, st, b_scores)));
      T_CK(launch(KID_ATTN_GENERIC, k_probs_from_lse, dim3(blocks256(n_sc)), dim3(256), 0, st, p.prob, (const float*)a.lse, (int)T,
                  att_scale, n_sc));
      T_CK((sgemm<0, 1>(p.dao, q, a.qkv + q + kv, nqkv, p.dsc, (int)T, (int)T, (int)T, hd, 0.f, st, b_dp)));     // dP = dO V^T
      T_CK(launch(KID_ATTN_GENERIC, k_attn_delta, dim3((unsigned)(M * hq)), dim3(64), 0, st, (const float*)p.dao, (const float*)a.ao,
                  (int)T, hq, hd, p.delta));
      T_CK(launch(KID_ATTN_GENERIC, k_dscores, dim3(blocks256(n_sc)), dim3(256), 0, st, (const float*)p.prob, p.dsc,
                  (const float*)p.delta, (int)T, att_scale, n_sc));
      T_CK((sgemm<0, 0>(p.dsc, (int)T, a.qkv + q, nqkv, p.dqkv, nqkv, (int)T, hd, (int)T, 0.f, st, b_dq)));       // dQ = dS K
      const bool one_launch = T % 16 == 0 && hd % 4 == 0 && nqkv % 4 == 0 && q % 4 == 0 && (long)T * hd * S_ * hkv >= 128 * 128;
      if (one_launch) {   // the query heads of a group are segments of one contraction (added in head order)
        Batch kd = b_dk, vd = b_dv;
        kd.kseg = vd.kseg = (int)T;
        kd.sega = vd.sega = TT;
        kd.segb = vd.segb = hd;
        T_CK((sgemm<1, 0>(p.dsc, (int)T, a.qkv, nqkv, p.dqkv + q, nqkv, (int)T, hd, rep * (int)T, 0.f, st, kd)));        // dK = sum_h dS_h^T Q_h
        T_CK((sgemm<1, 0>(p.prob, (int)T, p.dao, q, p.dqkv + q + kv, nqkv, (int)T, hd, rep * (int)T, 0.f, st, vd)));     // dV = sum_h P_h^T dO_h
      }
      for (int hh = 0; hh < (one_launch ? 0 : rep); ++hh) {   // otherwise one launch per head of the group, in order
        const float beta = hh > 0 ? 1.f : 0.f;
        T_CK((sgemm<1, 0>(p.dsc + (size_t)hh * T * T, (int)T, a.qkv + (size_t)hh * hd, nqkv, p.dqkv + q, nqkv, (int)T, hd, (int)T,
                          beta, st, b_dk)));                                                                       // dK += dS^T Q
        T_CK((sgemm<1, 0>(p.prob + (size_t)hh * T * T, (int)T, p.dao + (size_t)hh * hd, q, p.dqkv + q + kv, nqkv, (int)T, hd,
                          (int)T, beta, st, b_dv)));                                                               // dV += P^T dO
      }
    }
    {
      const size_t total = M * (size_t)(hq + hkv) * (hd / 2);
      T_CK(launch(KID_ROPE_APPEND, k_rope, dim3(blocks256(total)), dim3(256), 0, st, p.dqkv, (const float2*)tr->rope, (int)T,
                  hq + hkv, hd, nqkv, -1.0f, total));
    }
    if (tr->use_bias) {   // the biases enter before the rotary embedding: their gradient is the column sum of dqkv here
      T_CK(launch(KID_MISC, k_colsum_partial, dim3((nqkv + 255) / 256, n_gpart), dim3(256), 0, st, (const float*)p.dqkv, Mi, nqkv,
                  p.gpart));
      T_CK(launch(KID_MISC, k_gain_grad_finish, dim3((nqkv + 255) / 256), dim3(256), 0, st, (const float*)p.gpart, n_gpart, nqkv,
                  GR(tr->n_in + l)));
    }
    // query / key / value projections
    T_CK(mm_nn(p.dqkv, nqkv, TH(t0 + 1), d, p.dx, d, Mi, d, nqkv, 0.f));
    T_CK(mm_tn(p.dqkv, nqkv, a.xn, d, GR(t0 + 1), nqkv, d, Mi, 1.f));
    T_CK(norm_bwd(p.dx, a.h, a.r1, t0, 1));
  }
  T_CK(launch(KID_EMBED, k_embed_bwd, dim3(512), dim3(256), 0, st, tokens, (const float*)p.dh, Mi, d, V, GR(0)));

  return SAPO_OK;
}

extern "C" int sapo_policy_update(sapo_trainer* tr, const int32_t* tokens, const uint8_t* completion_mask,
                                  const float* logp_old, const float* advantages, int S_, int T_, float eps_low,
                                  float eps_high, float* out_loss, float* out_logp_new, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  if (!tr || !tokens || !completion_mask || !logp_old || !advantages || !out_loss || !workspace)
    return set_error(SAPO_EINVAL, "NULL argument");
  if (S_ <= 0 || T_ < 2) return set_error(SAPO_EINVAL, "S must be positive and T at least 2");
  if (T_ > tr->cfg.max_seq) return set_error(SAPO_EINVAL, "T = %d exceeds max_seq = %d", T_, tr->cfg.max_seq);
  if (T_ > 8192) return set_error(SAPO_EINVAL, "at most 8192 tokens per sequence");
  if (!(eps_low >= 0.f && eps_low < 1.f) || !(eps_high >= 0.f)) return set_error(SAPO_EINVAL, "eps_low in [0, 1), eps_high >= 0");
  const sapo_model_config& c = tr->cfg;
  const Dims D(c);
  const size_t S = S_, T = T_, M = S * T;
  if (M >= ((size_t)1 << 30)) return set_error(SAPO_EINVAL, "batch too large");
  // Micro-batches: the largest number of sequences whose activations fit the workspace is pushed through forward
  // and backward at a time, the gradients adding up; the whole set at once when the workspace allows it.
  TrainPlan p;
  size_t S_mb = S;
  // grid limits: sequences per launch of the fused attention kernels, (sequence, query head) pairs of a batched GEMM
  const size_t most = fused_attention(c) ? (size_t)65535 : (size_t)65535 / c.n_q_heads;
  if (S_mb > most) S_mb = most;
  make_plan(c, S_mb, T, S, nullptr, p);
  if (workspace_bytes < p.bytes) {
    size_t lo = 0, hi = S_mb;   // plan(lo) fits (lo = 0: nothing known to fit), plan(hi) does not
    while (hi - lo > 1) {
      const size_t mid = (lo + hi) / 2;
      make_plan(c, mid, T, S, nullptr, p);
      if (p.bytes <= workspace_bytes) lo = mid; else hi = mid;
    }
    if (lo == 0) {
      make_plan(c, 1, T, S, nullptr, p);
      return set_error(SAPO_EWORKSPACE, "workspace is %zu bytes, at least %zu needed (one sequence at a time)", workspace_bytes,
                       p.bytes);
    }
    S_mb = lo;
  }
  make_plan(c, S_mb, T, S, (char*)workspace, p);
  hipStream_t st = (hipStream_t)stream;
  const int t_head = c.tied_embeddings ? 0 : 1 + 9 * c.n_layers + 1;
  const int d = (int)D.d, V = (int)D.V;
  T_CK(g_fill_f32(tr->grad, 0.f, tr->n_params, st));
  T_CK(launch(KID_MISC, k_count_mask, dim3(1), dim3(256), 0, st, completion_mask, M, p.n_masked));
  T_CK(x3_pack(X3Op{tr->theta + tr->off[t_head], d, V, d, false}, p.head_nt, p.head_cap, tr->pieces, st));   // rows = vocabulary
  T_CK(x3_pack(X3Op{tr->theta + tr->off[t_head], d, d, V, true}, p.head_t, p.head_t_cap, tr->pieces, st));    // rows = d
  // The rows that predict a masked token, per micro-batch (indices within it, ascending), and how many there are:
  // the host needs the numbers to size the LM head's GEMMs, so the call waits here once, before the forward passes
  // are enqueued, for these small kernels (and for whatever the stream held before).
  const size_t n_mb = (S + S_mb - 1) / S_mb;
  std::vector<int> n_rows(n_mb, 0);
  for (size_t i = 0; i < n_mb; ++i) {
    const size_t s0 = i * S_mb;
    const int n = (int)(S - s0 < S_mb ? S - s0 : S_mb);
    T_CK(g_masked_rows(completion_mask + s0 * T, T_, 0, n, p.mpos, p.mrows + s0 * T, p.mcount + i, st));
  }
  T_CK(hipMemcpyAsync(n_rows.data(), p.mcount, n_mb * sizeof(int), hipMemcpyDeviceToHost, st));
  T_CK(hipStreamSynchronize(st));
  for (size_t i = 0; i < n_mb; ++i) {
    const size_t s0 = i * S_mb;
    const int n = (int)(S - s0 < S_mb ? S - s0 : S_mb);
    if (n_rows[i] < 0 || (size_t)n_rows[i] > (size_t)n * T) return set_error(SAPO_EHIP, "row count read back from the device is out of range");
    const int rc = update_rows(tr, p, tokens + s0 * T, completion_mask + s0 * T, logp_old + s0 * T, advantages + s0, n, T_,
                               eps_low, eps_high, p.logp_all + s0 * T, p.mrows + s0 * T, n_rows[i], st);
    if (rc != SAPO_OK) return rc;
  }
  // ---- the loss (the surrogate of sapo_clipped_surrogate on the log-probs just computed)
  T_CK(g_surrogate_loss(p.logp_all, logp_old, completion_mask, advantages, S_, T_, eps_low, eps_high, p.loss, nullptr, p.sur_ws,
                        st));
  T_CK(hipMemcpyAsync(out_loss, p.loss, sizeof(float), hipMemcpyDeviceToDevice, st));
  if (out_logp_new) T_CK(hipMemcpyAsync(out_logp_new, p.logp_all, M * sizeof(float), hipMemcpyDeviceToDevice, st));

  // ---- Adam
  tr->t += 1;
  const float c1 = (float)(1.0 - pow((double)tr->opt.beta1, (double)tr->t));
  const float c2 = (float)(1.0 - pow((double)tr->opt.beta2, (double)tr->t));
  T_CK(launch(KID_MISC, k_adam, dim3(blocks256(tr->n_params)), dim3(256), 0, st, tr->theta, (const float*)tr->grad, tr->m, tr->v,
              tr->n_params, tr->opt.lr, tr->opt.beta1, tr->opt.beta2, tr->opt.eps, c1, c2));
  return SAPO_OK;
}
