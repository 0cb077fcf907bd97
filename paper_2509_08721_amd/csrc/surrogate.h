// One token's term of the clipped surrogate (Sec. 4.2: GRPO without a KL term, asymmetric clipping), shared by
// the loss kernels and the policy update's LM-head pass so that both take the same branch for every token.
#pragma once
#include <hip/hip_runtime.h>

namespace sapo {

// term = min(rho A, clip(rho, 1 - eps_low, 1 + eps_high) A) with rho = exp(ln - lo); `active` says whether the
// unclipped branch is the minimum (then d term / d ln = rho A, else 0).
__device__ __forceinline__ float surrogate_term(float ln, float lo, float a, float eps_low, float eps_high, float& rho,
                                                bool& active) {
  rho = expf(ln - lo);
  const float clipped = fminf(fmaxf(rho, 1.0f - eps_low), 1.0f + eps_high);
  active = a >= 0.f ? (rho <= 1.0f + eps_high) : (rho >= 1.0f - eps_low);
  return fminf(rho * a, clipped * a);
}
// d loss / d ln for a masked token, the loss being -(sum of terms) / n_masked
__device__ __forceinline__ float surrogate_dlogp(float a, float rho, bool active, long long n_masked) {
  return active ? (float)(-(double)a * (double)rho / (double)n_masked) : 0.f;
}

}  // namespace sapo
