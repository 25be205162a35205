// Attention for launches that cover one in-block position t of every candidate (token-by-token generation).
// The prefix keys, shared by the n candidates of a beam, are handled by the MFMA kernel in its split mode, which
// stacks the n*g query rows of a (beam, kv head) and leaves per-split partial results (O un-normalised, running
// maximum m in the log2 domain, weight sum l). This file merges them with the candidate's own block keys
// 0..t (at most a block length of them): one wavefront per (candidate, query head).
#include "common.h"

bool launch_attention_mfma_decode_prefix(const bf16_t* q, const bf16_t* poolK, const bf16_t* poolV, const BatchGeom& g,
                                         const ModelDims& md, int max_ctx, float* part, size_t part_floats,
                                         int* q_tiles_out, int* n_splits_out, hipStream_t s);

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// hd % 8 == 0, Lp % 8 == 0 (block values are stored transposed and zero padded to Lp columns)
__global__ void __launch_bounds__(64) attention_decode_merge_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kb, const bf16_t* __restrict__ vbT,
    const float* __restrict__ part_o, const float* __restrict__ part_m, const float* __restrict__ part_l,
    bf16_t* __restrict__ out, int n, int Hq, int Hkv, int hd, int Lk, int Lp, int t, int q_tiles, int n_splits,
    float scale_log2e) {
  extern __shared__ float sm[];                 // [hd] query, [Lp] block scores then weights, [n_splits] split weights
  float* qs = sm;
  float* sc = sm + hd;
  float* wsplit = sc + Lp;
  const int c = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int g = Hq / Hkv, kvh = h / g, j = h - kvh * g;
  const int b = c / n, i = c - b * n;
  const int r = i * g + j, qt = r >> 7, rin = r & 127;
  const size_t prow0 = (((size_t)b * Hkv + kvh) * q_tiles + qt) * n_splits * 128 + rin;   // + split*128

  const bf16_t* qr = q + ((size_t)c * Hq + h) * hd;
  for (int d = lane; d < hd; d += 64) qs[d] = (float)qr[d];
  for (int jk = lane; jk < Lp; jk += 64) sc[jk] = 0.f;
  __syncthreads();
  // the candidate's own keys 0..t
  float mx = -INFINITY;
  for (int jk = lane; jk <= t; jk += 64) {
    const bf16_t* kr = kb + (((size_t)c * Lk + jk) * Hkv + kvh) * hd;
    float dot = 0.f;
    for (int d8 = 0; d8 < hd; d8 += 8) {
      bf16x8 kv = *(const bf16x8*)(kr + d8);
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(qs[d8 + e], (float)kv[e], dot);
    }
    dot *= scale_log2e;
    sc[jk] = dot;
    mx = fmaxf(mx, dot);
  }
  for (int s = lane; s < n_splits; s += 64) mx = fmaxf(mx, part_m[prow0 + (size_t)s * 128]);
  mx = wave_max(mx);                            // finite: key t itself is always visible
  float l = 0.f;
  for (int jk = lane; jk <= t; jk += 64) {
    float p = __builtin_amdgcn_exp2f(sc[jk] - mx);
    l += p;
    sc[jk] = (float)(bf16_t)p;                  // the weight that multiplies V is a bf16 operand
  }
  for (int s = lane; s < n_splits; s += 64) {
    float w = __builtin_amdgcn_exp2f(part_m[prow0 + (size_t)s * 128] - mx);   // exp2(-inf) = 0 for an empty split
    wsplit[s] = w;
    l += w * part_l[prow0 + (size_t)s * 128];
  }
  l = wave_sum(l);
  __syncthreads();
  const float inv = 1.0f / l;
  const int t8 = (t + 8) & ~7;                  // columns 0 .. t rounded up to whole 16-byte groups
  for (int d = lane; d < hd; d += 64) {
    float acc0 = 0.f, acc1 = 0.f;
    int s = 0;
    for (; s + 1 < n_splits; s += 2) {
      acc0 = fmaf(wsplit[s], part_o[(prow0 + (size_t)s * 128) * hd + d], acc0);
      acc1 = fmaf(wsplit[s + 1], part_o[(prow0 + (size_t)(s + 1) * 128) * hd + d], acc1);
    }
    if (s < n_splits) acc0 = fmaf(wsplit[s], part_o[(prow0 + (size_t)s * 128) * hd + d], acc0);
    const bf16_t* vr = vbT + (((size_t)c * Hkv + kvh) * hd + d) * Lp;
    for (int jk = 0; jk < t8; jk += 8) {
      bf16x8 vv = *(const bf16x8*)(vr + jk);
#pragma unroll
      for (int e = 0; e < 8; ++e)                 // columns beyond t hold whatever an earlier call left there
        acc0 = fmaf(sc[jk + e], jk + e <= t ? (float)vv[e] : 0.f, acc0);
    }
    out[((size_t)c * Hq + h) * hd + d] = (bf16_t)((acc0 + acc1) * inv);
  }
}

// Returns false when the shape is not taken (the caller then uses the plain kernel).
bool launch_attention_decode(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* poolK,
                             const bf16_t* poolV, bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp,
                             int max_ctx, float* part, size_t part_floats, hipStream_t s) {
  int q_tiles = 0, n_splits = 0;
  if (!launch_attention_mfma_decode_prefix(q, poolK, poolV, g, md, max_ctx, part, part_floats, &q_tiles, &n_splits, s))
    return false;
  int base = g.B * md.Hkv * q_tiles;
  size_t rows_all = (size_t)base * n_splits * 128;
  const float* part_m = part + rows_all * md.hd;
  const float* part_l = part_m + rows_all;
  size_t lds = (size_t)(md.hd + Lp + n_splits) * sizeof(float);
  float scale_log2e = 1.4426950408889634f / sqrtf((float)md.hd);
  attention_decode_merge_kernel<<<dim3(g.B * g.n, md.Hq), 64, lds, s>>>(q, kb, vbT, part, part_m, part_l, out, g.n,
                                                                       md.Hq, md.Hkv, md.hd, g.Lk, Lp, g.t0, q_tiles,
                                                                       n_splits, scale_log2e);
  return true;
}
