// Ancestral sampling of one token per row (Alg. 1, Step I): y = min{k : c_k > u * c_V}, c_k the running sum of
// exp(z_v - max z) over vocabulary ids v <= k, i.e. the inverse distribution function of the full softmax in id
// order, read at a uniform u supplied by the caller. Two kernels. The first cuts the ids into 128 chunks and
// leaves, per (row, chunk), the chunk's maximum and its sum of exp(z - chunk max) in double. The second, one block
// per row, rescales the chunk sums to the row maximum, scans them in id order to find the chunk in which the
// running sum crosses the threshold, and repeats the same scan-and-locate inside that chunk over per-thread runs
// and finally over single ids. All sums run in id order; only the grouping of the additions differs from one
// long running sum.
#include "common.h"
#include <climits>

constexpr int SAMPLE_CHUNKS = 128;

__device__ __forceinline__ double block_scan_256(double v, double* buf) {   // inclusive scan, buf[256]
  const int tid = threadIdx.x;
  buf[tid] = v;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    double add = tid >= off ? buf[tid - off] : 0.0;
    __syncthreads();
    buf[tid] += add;
    __syncthreads();
  }
  return buf[tid];
}

__global__ void __launch_bounds__(256) sample_chunks_kernel(const float* __restrict__ logits, int V, int limit,
                                                            float* __restrict__ cmax, double* __restrict__ csum) {
  __shared__ float wmax[4];
  __shared__ double wsum[4];
  const size_t row = blockIdx.x;
  const int chunk = blockIdx.y, tid = threadIdx.x;
  const int CH = (limit + SAMPLE_CHUNKS - 1) / SAMPLE_CHUNKS;
  const int c0 = chunk * CH, c1 = min(limit, c0 + CH);
  const float* z = logits + row * (size_t)V;
  const int run = (CH + 255) / 256;
  const int k0 = c0 + tid * run, k1 = min(c1, k0 + run);
  float mx = -INFINITY;
  for (int k = k0; k < k1; ++k) mx = fmaxf(mx, z[k]);
  mx = wave_max(mx);
  if ((tid & 63) == 0) wmax[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
  double sm = 0.0;
  if (mx > -INFINITY)
    for (int k = k0; k < k1; ++k) sm += exp((double)z[k] - (double)mx);
  // thread order = id order: add the wavefront's lanes in order, then the four wavefronts
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    double other = __shfl_up(sm, o, 64);
    if ((tid & 63) >= o) sm += other;
  }
  if ((tid & 63) == 63) wsum[tid >> 6] = sm;
  __syncthreads();
  if (tid == 0) {
    cmax[row * SAMPLE_CHUNKS + chunk] = mx;
    csum[row * SAMPLE_CHUNKS + chunk] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
  }
}

__global__ void __launch_bounds__(256) sample_pick_kernel(const float* __restrict__ logits, int V, int limit,
                                                          const float* __restrict__ cmax,
                                                          const double* __restrict__ csum,
                                                          const double* __restrict__ u, int32_t* __restrict__ cand,
                                                          float* __restrict__ tok_logp, int L, int t, int* status) {
  __shared__ double buf[256];
  __shared__ float wmax[4];
  __shared__ int sel;
  const size_t row = blockIdx.x;
  const int tid = threadIdx.x;
  const float* z = logits + row * (size_t)V;
  const int CH = (limit + SAMPLE_CHUNKS - 1) / SAMPLE_CHUNKS;

  float mx = tid < SAMPLE_CHUNKS ? cmax[row * SAMPLE_CHUNKS + tid] : -INFINITY;
  mx = wave_max(mx);
  if ((tid & 63) == 0) wmax[tid >> 6] = mx;
  if (tid == 0) sel = INT_MAX;
  __syncthreads();
  mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
  const double m = (double)mx;
  double w = 0.0;
  if (tid < SAMPLE_CHUNKS) {
    float cm = cmax[row * SAMPLE_CHUNKS + tid];
    if (cm > -INFINITY) w = csum[row * SAMPLE_CHUNKS + tid] * exp((double)cm - m);
  }
  double incl = block_scan_256(w, buf);
  const double total = buf[255];
  const double uu = u[row * L + t];
  const double thr = uu * total;
  const bool bad_u = !(uu >= 0.0 && uu < 1.0);
  const bool bad_z = !(total > 0.0) || !(total < INFINITY) || !(mx > -INFINITY);
  if (bad_u || bad_z) {
    if (tid == 0) {
      report_status(status, bad_u ? SPECS_ERANGE : SPECS_ENONFINITE);
      cand[row * L + t] = 0;
      tok_logp[row * L + t] = -INFINITY;
    }
    return;
  }
  // First chunk OF POSITIVE WEIGHT whose inclusive sum exceeds the threshold; none (rounding) -> the last chunk of
  // positive weight. The scan adds the same terms in a different grouping for every position, so its values need
  // not be monotone to the last bit: "first" is taken as a minimum over the threads that qualify (an LDS atomic),
  // never as "the one whose predecessor does not qualify", which may hold for several threads or for a chunk of
  // zero weight beyond the permitted ids.
  if (w > 0.0 && incl > thr) atomicMin(&sel, tid);
  __syncthreads();
  if (sel == INT_MAX) {
    if (tid == 0) {
      int c = SAMPLE_CHUNKS - 1;
      while (c > 0 && !(buf[c] > buf[c - 1])) --c;
      sel = c;
    }
    __syncthreads();
  }
  const int chunk = sel;
  const double before = chunk ? buf[chunk - 1] : 0.0;
  __syncthreads();                                     // buf is reused below
  // the same scan inside the chunk, over per-thread runs of ids
  const int c0 = chunk * CH, c1 = min(limit, c0 + CH);
  const int run = (CH + 255) / 256;
  const int k0 = c0 + tid * run, k1 = min(c1, k0 + run);
  double mine = 0.0;
  for (int k = k0; k < k1; ++k) mine += exp((double)z[k] - m);
  incl = block_scan_256(mine, buf) + before;
  const double excl = (tid ? buf[tid - 1] : 0.0) + before;
  __shared__ int first;
  if (tid == 0) { sel = -1; first = INT_MAX; }
  __syncthreads();
  if (mine > 0.0 && incl > thr) atomicMin(&first, tid);       // the first run that crosses the threshold, as above
  __syncthreads();
  if (tid == first) {
    double c = excl;
    int pick = -1;
    for (int k = k0; k < k1; ++k) {
      c += exp((double)z[k] - m);
      if (c > thr) { pick = k; break; }
    }
    if (pick < 0)
      for (int k = k1 - 1; k >= k0; --k)
        if (exp((double)z[k] - m) > 0.0) { pick = k; break; }
    sel = pick;
  }
  __syncthreads();
  if (tid == 0) {
    int pick = sel;
    if (pick < 0)                                      // threshold not exceeded inside the chunk: its last id of positive weight
      for (int k = c1 - 1; k >= c0; --k)
        if (exp((double)z[k] - m) > 0.0) { pick = k; break; }
    if (pick < 0) pick = c0;
    cand[row * L + t] = pick;
    tok_logp[row * L + t] = (float)((double)z[pick] - m - log(total));
  }
}

size_t sample_scratch_bytes(int rows) { return (size_t)rows * SAMPLE_CHUNKS * (sizeof(double) + sizeof(float)); }

// scratch: sample_scratch_bytes(rows) bytes, 8-byte aligned
void launch_sample_tokens(const float* logits, int rows, int V, int limit, const double* u, int32_t* cand,
                          float* tok_logp, int L, int t, void* scratch, int* status, hipStream_t s) {
  double* csum = (double*)scratch;
  float* cmax = (float*)(csum + (size_t)rows * SAMPLE_CHUNKS);
  sample_chunks_kernel<<<dim3(rows, SAMPLE_CHUNKS), 256, 0, s>>>(logits, V, limit, cmax, csum);
  sample_pick_kernel<<<rows, 256, 0, s>>>(logits, V, limit, cmax, csum, u, cand, tok_logp, L, t, status);
}
