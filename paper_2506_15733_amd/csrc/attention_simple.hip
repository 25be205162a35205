// Straightforward shared-prefix attention: one wavefront per (row, query head). Serves the float
// configuration, head sizes the MFMA kernel does not take, and launches that cover one in-block position of every
// candidate (row m = candidate m / L at position t0 + m % L; its block keys are rows cand*Lk .. of kb). Three passes over the keys:
// scores into LDS (+ max), un-normalised weights 2^(s' - ceil(max s')) in the log2 domain (+ sum; the integer
// reference makes the bf16 rounding of the weights independent of which power of two they are scaled by), weighted
// sum of V.
#include "common.h"

template <typename T>
__global__ void __launch_bounds__(64) attention_simple_kernel(const T* __restrict__ q, const T* __restrict__ kb,
                                                              const T* __restrict__ vbT, const T* __restrict__ poolK,
                                                              const T* __restrict__ poolV, T* __restrict__ out,
                                                              BatchGeom g, int Hq, int Hkv, int hd, int Lp, float scale) {
  extern __shared__ float sc[];                 // [ctx + t + 1] scores, then weights
  int m = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  int nL = g.n * g.L;
  int b = m / nL, t = g.t0 + m % g.L;               // in-block position of this row
  int ctx = g.len_override >= 0 ? g.len_override : g.lens[g.b0 + b];
  int kvh = h / (Hq / Hkv);
  int nkeys = ctx + t + 1;
  const T* qr = q + ((size_t)m * Hq + h) * hd;
  const int32_t* pt = g.page_table + (size_t)(g.b0 + b) * g.max_pages;
  float* qs = sc + nkeys;                       // [hd] query staged in LDS as float
  for (int c = lane; c < hd; c += 64) qs[c] = to_f32<T>(qr[c]);
  __syncthreads();

  float mx = -INFINITY;
  for (int j = lane; j < nkeys; j += 64) {
    const T* kr;
    if (j < ctx) {
      int page = pt[j / g.page_tokens], slot = j % g.page_tokens;
      kr = poolK + (((size_t)page * Hkv + kvh) * g.page_tokens + slot) * hd;
    } else {
      kr = kb + (((size_t)(m / g.L) * g.Lk + (j - ctx)) * Hkv + kvh) * hd;
    }
    float dot = 0.f;
    for (int c = 0; c < hd; ++c) dot = fmaf(qs[c], to_f32<T>(kr[c]), dot);
    dot *= scale;                                // scale = log2(e) / sqrt(hd): scores in the log2 domain
    sc[j] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = ceilf(wave_max(mx));
  float sm = 0.f;
  for (int j = lane; j < nkeys; j += 64) {
    float p = exp2f(sc[j] - mx);
    sm += p;
    sc[j] = to_f32<T>(from_f32<T>(p));          // the weight that multiplies V is an operand: rounded to T
  }
  sm = wave_sum(sm);
  __syncthreads();
  float inv = 1.0f / sm;
  // values are stored transposed: pages [page][Hkv][hd][pt], block [cand][Hkv][hd][Lp]
  size_t cand = (size_t)(m / g.L);
  for (int c = lane; c < hd; c += 64) {
    float acc = 0.f;
    const T* vblk = vbT + ((cand * Hkv + kvh) * hd + c) * Lp;
    for (int j = 0; j < nkeys; ++j) {
      float vv;
      if (j < ctx) {
        int page = pt[j / g.page_tokens], slot = j % g.page_tokens;
        vv = to_f32<T>(poolV[(((size_t)page * Hkv + kvh) * hd + c) * g.page_tokens + slot]);
      } else {
        vv = to_f32<T>(vblk[j - ctx]);
      }
      acc = fmaf(sc[j], vv, acc);
    }
    out[((size_t)m * Hq + h) * hd + c] = from_f32<T>(acc * inv);
  }
}

template <typename T>
void launch_attention_simple(const T* q, const T* kb, const T* vbT, const T* poolK, const T* poolV, T* out,
                             const BatchGeom& g, const ModelDims& md, int Lp, int max_ctx, hipStream_t s) {
  size_t lds = (size_t)(max_ctx + g.Lk + md.hd) * sizeof(float);
  float scale = 1.4426950408889634f / sqrtf((float)md.hd);
  (void)hipFuncSetAttribute((const void*)attention_simple_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  attention_simple_kernel<T><<<dim3(g.M, md.Hq), 64, lds, s>>>(q, kb, vbT, poolK, poolV, out, g, md.Hq, md.Hkv, md.hd,
                                                               Lp, scale);
}
template void launch_attention_simple<float>(const float*, const float*, const float*, const float*, const float*,
                                             float*, const BatchGeom&, const ModelDims&, int, int, hipStream_t);
template void launch_attention_simple<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, const bf16_t*,
                                              const bf16_t*, bf16_t*, const BatchGeom&, const ModelDims&, int, int,
                                              hipStream_t);
