// Ancestral sampling of one token per row (Alg. 1, Step I): y = min{k : c_k > u * c_V}, c_k the running sum of
// exp(z_v - max z) over vocabulary ids v <= k, i.e. the inverse distribution function of the full softmax in id
// order, read at a uniform u supplied by the caller. One 1024-thread block per row; every thread owns one
// contiguous run of ids, sums it sequentially in double, a block-wide scan of the 1024 run sums locates the run
// that crosses the threshold, and its owner walks it again to find the id. Sums are therefore taken in id order
// (run by run), as the definition states; only the grouping of the additions differs from a single running sum.
#include "common.h"

__global__ void __launch_bounds__(1024) sample_tokens_kernel(const float* __restrict__ logits, int V, int limit,
                                                             const double* __restrict__ u, int32_t* __restrict__ cand,
                                                             float* __restrict__ tok_logp, int L, int t, int* status) {
  __shared__ double incl[1024];
  __shared__ float wmax[16];
  __shared__ int found;
  const size_t row = blockIdx.x;
  const float* z = logits + row * (size_t)V;
  const int tid = threadIdx.x;
  const int run = (limit + 1023) / 1024;
  const int k0 = tid * run, k1 = min(limit, k0 + run);

  float mx = -INFINITY;
  for (int k = k0; k < k1; ++k) mx = fmaxf(mx, z[k]);
  mx = wave_max(mx);
  if ((tid & 63) == 0) wmax[tid >> 6] = mx;
  if (tid == 0) found = -1;
  __syncthreads();
  mx = wmax[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) mx = fmaxf(mx, wmax[w]);
  const double m = (double)mx;

  double mine = 0.0;
  for (int k = k0; k < k1; ++k) mine += exp((double)z[k] - m);
  incl[tid] = mine;
  __syncthreads();
  // inclusive scan over the 1024 run sums (Hillis-Steele)
  for (int off = 1; off < 1024; off <<= 1) {
    double add = tid >= off ? incl[tid - off] : 0.0;
    __syncthreads();
    incl[tid] += add;
    __syncthreads();
  }
  const double total = incl[1023];
  const double uu = u[row * L + t];
  const double thr = uu * total;
  const bool bad_u = !(uu >= 0.0 && uu < 1.0);
  const bool bad_z = !(total > 0.0) || !(total < INFINITY) || !(mx > -INFINITY);
  if (tid == 0 && (bad_u || bad_z)) *status = bad_u ? SPECS_ERANGE : SPECS_ENONFINITE;
  if (!bad_u && !bad_z) {
    const double before = tid ? incl[tid - 1] : 0.0;
    if (incl[tid] > thr && !(before > thr)) {           // the first run whose inclusive sum exceeds the threshold
      double c = before;
      int pick = -1;
      for (int k = k0; k < k1; ++k) {
        c += exp((double)z[k] - m);
        if (c > thr) { pick = k; break; }
      }
      if (pick < 0)                                      // rounding between the two passes: last id of positive weight
        for (int k = k1 - 1; k >= k0; --k)
          if (exp((double)z[k] - m) > 0.0) { pick = k; break; }
      found = pick;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int pick = found;
    if (pick < 0 && !bad_u && !bad_z)                    // threshold not exceeded anywhere: last id of positive weight
      for (int k = limit - 1; k >= 0; --k)
        if (exp((double)z[k] - m) > 0.0) { pick = k; break; }
    if (pick < 0) pick = 0;
    cand[row * L + t] = pick;
    tok_logp[row * L + t] = (bad_u || bad_z) ? -INFINITY : (float)((double)z[pick] - m - log(total));
  }
}

void launch_sample_tokens(const float* logits, int rows, int V, int limit, const double* u, int32_t* cand,
                          float* tok_logp, int L, int t, int* status, hipStream_t s) {
  sample_tokens_kernel<<<rows, 1024, 0, s>>>(logits, V, limit, u, cand, tok_logp, L, t, status);
}
