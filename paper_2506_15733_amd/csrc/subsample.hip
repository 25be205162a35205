// SubSample (Alg. 2): one 64-lane wavefront per (beam, beta). Scores (Eq. 1), their maximum and
// the maximum reward are wave reductions (exact, order-free); the cumulative sum of the
// max-shifted exponentials runs in index order in double so that, given the same scores and the
// same uniform, the chosen index is the one a sequential double-precision pass would choose.
#include "common.h"

struct BetaList { float v[SPECS_MAX_BETAS]; };

__device__ __forceinline__ double wave_max_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}

__global__ void __launch_bounds__(64) subsample_kernel(const float* __restrict__ lt, const float* __restrict__ lg,
                                                       const float* __restrict__ r, const uint8_t* __restrict__ mask,
                                                       int n, BetaList betas, int nb, const double* __restrict__ u,
                                                       int32_t* __restrict__ idx, float* __restrict__ max_reward,
                                                       uint8_t* __restrict__ gen_is_draft, float tau, int* status) {
  __shared__ double w[SPECS_MAX_CANDIDATES];
  int b = blockIdx.x, j = blockIdx.y, lane = threadIdx.x;
  double beta = (double)betas.v[j];
  // Alg. 1: while the target model generates a beam's blocks, pi_gen = pi_target and the log-ratio of Eq. 1 is 0
  const bool gen_target = gen_is_draft != nullptr && gen_is_draft[b] == 0;
  double smax = -INFINITY;
  float rmax = -INFINITY;
  bool bad = false;
  int live = 0;
  for (int i = lane; i < n; i += 64) {
    size_t o = (size_t)b * n + i;
    double S = (gen_target ? 0.0 : (double)lt[o] - (double)lg[o]) + beta * (double)r[o];
    bool on = mask ? mask[o] != 0 : true;
    rmax = fmaxf(rmax, r[o]);
    if (on) {
      if (!isfinite(S)) bad = true;
      smax = fmax(smax, S);
      ++live;
    }
    w[i] = on ? S : -INFINITY;
  }
  smax = wave_max_f64(smax);
  rmax = wave_max(rmax);
  bad = __any(bad);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) live += __shfl_xor(live, o, 64);
  for (int i = lane; i < n; i += 64) w[i] = (w[i] == -INFINITY) ? 0.0 : exp(w[i] - smax);
  __syncthreads();
  if (lane == 0) {
    if (j == 0 && max_reward) max_reward[b] = rmax;
    double uu = u[(size_t)b * nb + j];
    int pick = -1;
    if (bad || live == 0) {
      report_status(status, SPECS_ENONFINITE);
    } else if (!(uu >= 0.0 && uu < 1.0)) {
      report_status(status, SPECS_ERANGE);
    } else {
      double total = 0.0;
      for (int i = 0; i < n; ++i) total += w[i];
      double thr = uu * total, run = 0.0;
      for (int i = 0; i < n; ++i) {
        run += w[i];
        if (run > thr) { pick = i; break; }
      }
      if (pick < 0)
        for (int i = n - 1; i >= 0; --i)
          if (w[i] > 0.0) { pick = i; break; }
    }
    idx[(size_t)b * nb + j] = pick;
    // Alg. 1 Step III: once some candidate's reward exceeds the threshold (strictly), the draft model generates
    // this beam's blocks from the next iteration on, for good
    if (gen_is_draft != nullptr && j == 0 && rmax > tau) gen_is_draft[b] = 1;
  }
}

void launch_subsample(const float* lt, const float* lg, const float* r, const uint8_t* mask, int B, int n,
                      const float* beta_host, int nb, const double* u, int32_t* idx, float* max_reward,
                      uint8_t* gen_is_draft, float tau, int* status, hipStream_t s) {
  BetaList bl = {};
  for (int j = 0; j < nb; ++j) bl.v[j] = beta_host[j];
  subsample_kernel<<<dim3(B, nb), 64, 0, s>>>(lt, lg, r, mask, n, bl, nb, u, idx, max_reward, gen_is_draft, tau, status);
}
