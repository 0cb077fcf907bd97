// One decode step's layers as ONE persistent kernel (gfx950): up to 64 rows, one new token per row.
//
// A decode step of a small decoder is a chain of tiny dependent phases (per layer: QKV projection, attention,
// output projection, gate/up + SwiGLU, down projection), each moving a few MB of weights.  As one kernel per phase
// the chain pays, per phase, a launch ramp, a first trip to HBM for the weights that cannot start before the
// kernel does, and the cache write-back / invalidate of a kernel boundary.  Here one workgroup per compute unit
// stays resident for the whole step and walks the phases itself:
//   * weights do not depend on activations, so a workgroup requests the weight tiles of its next unit of work
//     BEFORE it waits for the previous phase: they arrive while it waits;
//   * what one phase hands to the next travels through memory with write-through stores and L2-bypassing loads
//     (decode_units.h, COH = true): no cache is written back or invalidated wholesale;
//   * the phases are separated by an exchange: every workgroup counts itself in when its stores have completed
//     (one counter per arrival group, 8 groups by block id modulo 8, which is the XCD under round-robin dispatch;
//     the last of a group adds to the global counter), and a consumer polls the global counter before it reads.
//     Counters only grow: the n-th launch since they were zeroed starts from n * (arrivals per launch), n being a
//     word the last workgroup to report a launch's last phase moves on, so nothing is reset between the replays of
//     the captured step.
// Every wait is bounded by a wall-clock limit: a workgroup that waits longer (its peers cannot all be resident,
// e.g. because other work holds compute units) sets the fault word, stops waiting for the rest of the launch and
// runs to the end; the sampler then emits -1 tokens, so the failure is visible and no wave is left spinning.
// Measured on the 0.5B-class decoder (64 rows) the kernel does NOT beat one kernel per phase: 815 us per launch against
// about 750 us for the same 120 phases as kernels (the hand-over between workgroups costs 3-4 us per phase, a kernel
// boundary in a replayed graph 2.3 us).  It is kept as an option (SAPO_PERSIST=1 in the environment), off by default.
// The arithmetic is that of the per-phase kernels (same device functions, same summation orders): a step through
// this kernel returns the same bytes.
#include "decode_units.h"

namespace sapo {

namespace {

constexpr int kGroups = 8;
constexpr size_t kRedBytes = 131072;                 // the largest cross-wave reduction buffer of a GEMM unit
constexpr size_t kPersistSmem = kRedBytes + 512 * sizeof(float);

#ifdef SAPO_PERSIST_TRACE
// Diagnostic build (-DSAPO_PERSIST_TRACE): per workgroup and phase type, summed over a run, the ticks of the 100 MHz
// wall clock from one report to the next, those spent waiting for the previous phase, those spent in the report
// (draining the stores, the barrier, the counters), and the number of phases.  Read with sapo_debug_persist_trace.
__device__ unsigned long long g_trace[256][5][4];
#endif

struct Exchange {
#ifdef SAPO_PERSIST_TRACE
  mutable unsigned long long t_prev = 0, t_wait = 0;
#endif
  PersistCtl* ctl;
  unsigned base_global, base_group;   // counter values when this launch began
  unsigned group_size;                // workgroups per arrival group
  int group;
  unsigned spin_ticks;
  int* s_dead;                        // LDS: a wait of this workgroup has timed out
  unsigned launch, n_phases;

  // all workgroups have reported `phases` phases (every thread of the workgroup calls this)
  __device__ __forceinline__ void wait_for(unsigned phases) const {
#ifdef SAPO_PERSIST_TRACE
    const unsigned long long tw0 = wall_clock64();
#endif
    if (threadIdx.x == 0 && *s_dead == 0) {
      const unsigned target = base_global + (unsigned)kGroups * phases;
      const unsigned long long t0 = wall_clock64();
      while ((int)(__hip_atomic_load(&ctl->global, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
        if (wall_clock64() - t0 > spin_ticks) {
          *s_dead = 1;
          atomicOr(&ctl->fault, 1u);
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    __syncthreads();
#ifdef SAPO_PERSIST_TRACE
    t_wait += wall_clock64() - tw0;
#endif
  }
  // this workgroup's part of phase number `phase` (0-based) is written (every thread calls this)
  __device__ __forceinline__ void arrive(unsigned phase) const {
#ifdef SAPO_PERSIST_TRACE
    const unsigned long long ta0 = wall_clock64();
#endif
    coh_drain();
    __syncthreads();
    const unsigned done = phase + 1u;
    if (threadIdx.x == 0) {
      const unsigned old = __hip_atomic_fetch_add(&ctl->group[group][0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old + 1u == base_group + group_size * done) {
        const unsigned og = __hip_atomic_fetch_add(&ctl->global, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the very last report of the launch: every workgroup has long read the launch index; the next launch reads
        // the new one after the kernel boundary
        if (og + 1u == base_global + (unsigned)kGroups * n_phases) ctl->launches = launch + 1u;
      }
    }
#ifdef SAPO_PERSIST_TRACE
    if (threadIdx.x == 0 && blockIdx.x < 256) {
      const unsigned long long now = wall_clock64();
      unsigned long long* t = g_trace[blockIdx.x][phase % 5];
      t[0] += now - t_prev; t[1] += t_wait; t[2] += now - ta0; t[3] += 1;
      t_prev = now; t_wait = 0;
    }
#endif
  }
};

// The units of one GEMM phase dealt to the resident workgroups.  Unit ids that differ by a multiple of 8 share a
// weight tile (they run on one XCD and the tile comes from HBM once).  need: phases that must be complete before
// the input may be read (0: the input comes from an earlier launch).
template <int NT, int TG, int R, int MODE>
__device__ __forceinline__ void gemm_phase(const SkinnyArgs& a, const Exchange& ex, unsigned need, char* smem) {
  constexpr int TS = 4 / TG;
  float4* red = (float4*)smem;
  float* s_part = (float*)(smem + kRedBytes);
  const int n_units = a.N / 16 / NT;
  const int total = (n_units + 7) / 8 * 8 * TS;
  bool first = true;
  for (int u = blockIdx.x; u < total; u += gridDim.x) {
    const int j = u >> 3;
    const int unit = (j / TS) * 8 + (u & 7);
    if (unit >= n_units) continue;
    if (!first) __syncthreads();   // the previous unit's epilogue has read the LDS buffers
    const bool wait_now = first && need > 0;
    skinny_unit<NT, TG, R, MODE, true>(a, unit, 0, (j % TS) * TG, red, s_part, [&]() { if (wait_now) ex.wait_for(need); });
    first = false;
  }
  // a workgroup without a unit waits too: reports of consecutive phases must not mix in a group's counter
  if (first && need > 0) ex.wait_for(need);
  ex.arrive(need);
}

template <int MODE>
__device__ __forceinline__ void gemm_phase_variant(int variant, const SkinnyArgs& a, const Exchange& ex, unsigned need, char* smem) {
  if constexpr (MODE == SKM_SWIGLU) {
    if (variant == 0) gemm_phase<4, 4, 4, SKM_SWIGLU>(a, ex, need, smem);
    else gemm_phase<2, 4, 6, SKM_SWIGLU>(a, ex, need, smem);
  } else {
    switch (variant) {
      case 0: gemm_phase<1, 1, 8, MODE>(a, ex, need, smem); break;
      case 1: gemm_phase<1, 2, 8, MODE>(a, ex, need, smem); break;
      default: gemm_phase<1, 1, 20, MODE>(a, ex, need, smem); break;
    }
  }
}

template <int HD, int PD>
__global__ void __launch_bounds__(512) k_decode_layers(PersistArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int s_dead;
  if (threadIdx.x == 0) s_dead = 0;
  __syncthreads();
  const unsigned launch = A.ctl->launches;
  const unsigned n_phases = 5u * (unsigned)A.n_layers;
  Exchange ex;
  ex.launch = launch;
  ex.n_phases = n_phases;
  ex.ctl = A.ctl;
  ex.group = blockIdx.x % kGroups;
  ex.group_size = gridDim.x / kGroups;
  ex.base_global = launch * (unsigned)kGroups * n_phases;
  ex.base_group = launch * ex.group_size * n_phases;
  ex.spin_ticks = A.spin_ticks;
  ex.s_dead = &s_dead;
#ifdef SAPO_PERSIST_TRACE
  ex.t_prev = wall_clock64();
#endif
  const int d = A.d, F = A.F, hkv = A.kv0.n_kv_heads;
  const int nqkv = A.q_dim + 2 * A.kv_dim;
  unsigned ph = 0;   // phases before the current one
  for (int l = 0; l < A.n_layers; ++l) {
    const PersistLayer L = A.layers[l];
    KVCache kvc = A.kv0;
    kvc.k = (char*)A.kv0.k + (size_t)l * A.kv_layer_stride;
    kvc.v = (char*)A.kv0.v + (size_t)l * A.kv_layer_stride;
    {   // QKV projection of the attention-normed residual
      SkinnyArgs a{};
      a.n_rows = A.S; a.s_pad = A.s_pad; a.eps = A.eps; a.norm_dim = d;
      a.Wp = L.wqkv; a.Xp = A.xa; a.N = nqkv; a.K = d;
      a.ssq_in = A.ssq_a; a.ssq_parts = (l == 0) ? 1 : d / 16;
      a.out_f32 = A.qkv; a.ldc = nqkv; a.bias = L.bqkv;
      gemm_phase_variant<SKM_STORE>(A.v_qkv, a, ex, ph, smem);
      ++ph;
    }
    {   // rotary, KV append, attention
      bool first = true;
      for (int u = blockIdx.x; u < A.S * hkv; u += gridDim.x) {
        const bool wait_now = first;
        attention_unit<HD, 8, PD, true>(A.qkv, A.rope, A.rm, kvc, A.attn, A.n_q_heads, u / hkv, u % hkv, smem,
                                        [&]() { if (wait_now) ex.wait_for(ph); });
        first = false;
      }
      if (first) ex.wait_for(ph);
      ex.arrive(ph);
      ++ph;
    }
    {   // output projection + residual; emits the FFN norm's operand
      SkinnyArgs a{};
      a.n_rows = A.S; a.s_pad = A.s_pad;
      a.Wp = L.wo; a.Xp = A.attn; a.N = d; a.K = A.q_dim;
      a.h = A.h; a.gain_next = L.ffn_norm; a.xp_out = A.xb; a.ssq_out = A.ssq_b;
      gemm_phase_variant<SKM_RESID>(A.v_o, a, ex, ph, smem);
      ++ph;
    }
    {   // gate / up projections + SwiGLU
      SkinnyArgs a{};
      a.n_rows = A.S; a.s_pad = A.s_pad; a.eps = A.eps; a.norm_dim = d;
      a.Wp = L.wgu; a.Xp = A.xb; a.N = 2 * F; a.K = d;
      a.ssq_in = A.ssq_b; a.ssq_parts = d / 16;
      a.xp_out = A.act;
      gemm_phase_variant<SKM_SWIGLU>(A.v_gu, a, ex, ph, smem);
      ++ph;
    }
    {   // down projection + residual; emits the next norm's operand
      SkinnyArgs a{};
      a.n_rows = A.S; a.s_pad = A.s_pad;
      a.Wp = L.wdown; a.Xp = A.act; a.N = d; a.K = F;
      a.h = A.h; a.gain_next = L.gain_after; a.xp_out = A.xa; a.ssq_out = A.ssq_a;
      gemm_phase_variant<SKM_RESID>(A.v_down, a, ex, ph, smem);
      ++ph;
    }
  }
}

// blocking of a STORE / RESID phase: 20 k steps per wave and round when 8 do not cover K (one 16-token group per
// unit: two would not fit the registers); otherwise two 16-token groups per unit when single groups would give more
// units than workgroups
int pick_variant(int N, int K, int n_wg) {
  const int tiles = N / 16, per_wave = (K / 32 + 7) / 8;
  if (per_wave > 8) return 2;
  return tiles * 4 > n_wg ? 1 : 0;
}

}  // namespace

#ifdef SAPO_PERSIST_TRACE
}  // namespace sapo
// out: 256 x 5 x 4 counters (see g_trace); reset != 0 clears them afterwards.  Diagnostic builds only.
extern "C" int sapo_debug_persist_trace(unsigned long long* out, int reset) {
  if (out && hipMemcpyFromSymbol(out, HIP_SYMBOL(sapo::g_trace), sizeof(sapo::g_trace)) != hipSuccess) return -1;
  if (reset) {
    static unsigned long long zeros[256 * 5 * 4];
    if (hipMemcpyToSymbol(HIP_SYMBOL(sapo::g_trace), zeros, sizeof(zeros)) != hipSuccess) return -1;
  }
  return 0;
}
namespace sapo {
#endif

size_t d_decode_layers_ctl_bytes() { return sizeof(PersistCtl); }

bool d_decode_layers_supported(int S, int d, int q_dim, int kv_dim, int F, int head_dim, int n_kv_heads) {
  if (S < 1 || S > 64) return false;
  if (head_dim != 64 && head_dim != 128) return false;
  if (d % 32 != 0 || q_dim % 32 != 0 || F % 32 != 0 || d % 16 != 0 || (q_dim + 2 * kv_dim) % 16 != 0) return false;
  if (d / 16 > 8 * kSsqPerThread) return false;        // sums-of-squares parts a GEMM unit can add up
  if ((2 * F / 16) % 4 != 0) return false;             // gate / up tiles come in pairs, 2 or 4 per unit
  // buffer instructions address below 2 GiB
  if ((size_t)64 * (size_t)(F > d ? F : d) * 4 >= ((size_t)1 << 31)) return false;
  return true;
}

namespace {
int g_persist_wgs = 0;   // workgroups of a launch: one per compute unit, a multiple of the arrival groups; 0: not prepared

template <typename K>
hipError_t prepare_kernel(K kernel) {
  hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPersistSmem);
  if (e != hipSuccess) return e;
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 512, kPersistSmem);
  if (e != hipSuccess) return e;
  return per_cu >= 1 ? hipSuccess : hipErrorLaunchOutOfResources;   // every workgroup must be resident at once
}
}  // namespace

// Once per process, outside any stream capture: kernel attributes, and the check that one workgroup fits a compute unit.
hipError_t d_decode_layers_prepare() {
  if (g_persist_wgs > 0) return hipSuccess;
  int dev = 0, n_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  if (n_cu < kGroups) return hipErrorInvalidValue;
  if ((e = prepare_kernel(k_decode_layers<64, 3>)) != hipSuccess) return e;
  if ((e = prepare_kernel(k_decode_layers<128, 2>)) != hipSuccess) return e;
  g_persist_wgs = n_cu / kGroups * kGroups;
  return hipSuccess;
}

hipError_t d_decode_layers(PersistArgs A, int head_dim, hipStream_t st) {
  if (g_persist_wgs <= 0) return hipErrorNotInitialized;
  const int n_wg = g_persist_wgs;
  A.v_qkv = pick_variant(A.q_dim + 2 * A.kv_dim, A.d, n_wg);
  A.v_o = pick_variant(A.d, A.q_dim, n_wg);
  A.v_down = pick_variant(A.d, A.F, n_wg);
  A.v_gu = ((A.d / 32 + 7) / 8 <= 4) ? 0 : 1;
  A.spin_ticks = 20000000u;   // 0.2 s of the 100 MHz wall clock
  if (head_dim == 64) return launch(KID_DECODE_LAYERS, k_decode_layers<64, 3>, dim3(n_wg), dim3(512), kPersistSmem, st, A);
  if (head_dim == 128) return launch(KID_DECODE_LAYERS, k_decode_layers<128, 2>, dim3(n_wg), dim3(512), kPersistSmem, st, A);
  return hipErrorInvalidValue;
}

}  // namespace sapo
