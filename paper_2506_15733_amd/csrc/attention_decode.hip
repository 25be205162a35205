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

// Lp % 8 == 0 (block values are stored transposed and padded to Lp columns). The kernel is a chain of short
// dependent phases, so every loop over memory is unrolled into batches of independent 16-byte loads.
template <int HD>
__global__ void __launch_bounds__(64) attention_decode_merge_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kb, const bf16_t* __restrict__ vbT,
    const float* __restrict__ part_o, const float* __restrict__ part_m, const float* __restrict__ part_l,
    bf16_t* __restrict__ out, int n, int Hq, int Hkv, int Lk, int Lp, int t, int q_tiles, int n_splits,
    float scale_log2e) {
  constexpr int hd = HD;
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
    bf16x8 kv[HD / 8];
#pragma unroll
    for (int i8 = 0; i8 < HD / 8; ++i8) kv[i8] = *(const bf16x8*)(kr + 8 * i8);
    float dot = 0.f;
#pragma unroll
    for (int i8 = 0; i8 < HD / 8; ++i8)
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(qs[8 * i8 + e], (float)kv[i8][e], dot);
    dot *= scale_log2e;
    sc[jk] = dot;
    mx = fmaxf(mx, dot);
  }
  for (int s = lane; s < n_splits; s += 64) mx = fmaxf(mx, part_m[prow0 + (size_t)s * 128]);
  mx = ceilf(wave_max(mx));                     // finite (key t itself is always visible); an integer, so that
                                                // the bf16 rounding of the weights does not depend on the reference
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
#pragma unroll
  for (int d = lane; d < HD; d += 64) {
    float acc = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += 8) {           // eight partial results at a time
      float po[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) po[k] = s0 + k < n_splits ? part_o[(prow0 + (size_t)(s0 + k) * 128) * HD + d] : 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = fmaf(s0 + k < n_splits ? wsplit[s0 + k] : 0.f, po[k], acc);
    }
    const bf16_t* vr = vbT + (((size_t)c * Hkv + kvh) * HD + d) * Lp;
    for (int j0 = 0; j0 < t8; j0 += 64) {                // eight 16-byte groups of block values at a time
      bf16x8 vv[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) vv[k] = j0 + 8 * k < t8 ? *(const bf16x8*)(vr + j0 + 8 * k) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) {                   // columns beyond t hold whatever an earlier call left there
          const int jk = j0 + 8 * k + e;
          acc = fmaf(jk <= t ? sc[jk] : 0.f, jk <= t ? (float)vv[k][e] : 0.f, acc);
        }
    }
    out[((size_t)c * Hq + h) * HD + d] = (bf16_t)(acc * inv);
  }
}

// The same merge for block buffers of at most 128 columns and at most 16 splits, with every load whose address
// does not depend on computed values (block keys, split statistics, partial outputs, block values) issued up front
// into registers, so that the kernel waits for memory once instead of once per phase.
template <int HD>
__global__ void __launch_bounds__(64) attention_decode_merge_fast_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kb, const bf16_t* __restrict__ vbT,
    const float* __restrict__ part_o, const float* __restrict__ part_m, const float* __restrict__ part_l,
    bf16_t* __restrict__ out, int n, int Hq, int Hkv, int Lk, int Lp, int t, int q_tiles, int n_splits,
    float scale_log2e) {
  constexpr int ND = HD / 64;                   // output dims per lane
  __shared__ float qs[HD];
  __shared__ float sc[128];
  __shared__ float wsplit[16];
  const int c = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int g = Hq / Hkv, kvh = h / g, j = h - kvh * g;
  const int b = c / n, i = c - b * n;
  const int r = i * g + j, qt = r >> 7, rin = r & 127;
  const size_t prow0 = (((size_t)b * Hkv + kvh) * q_tiles + qt) * n_splits * 128 + rin;
  const int t8 = (t + 8) & ~7;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  // ---- all loads
  const bf16_t* qr = q + ((size_t)c * Hq + h) * HD;
  float qv[ND];
#pragma unroll
  for (int u = 0; u < ND; ++u) qv[u] = (float)qr[lane + 64 * u];
  bf16x8 kv[2][HD / 8];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int jk = lane + 64 * kk;
    const bf16_t* kr = kb + (((size_t)c * Lk + (jk <= t ? jk : t)) * Hkv + kvh) * HD;
#pragma unroll
    for (int i8 = 0; i8 < HD / 8; ++i8) kv[kk][i8] = *(const bf16x8*)(kr + 8 * i8);
  }
  float pm = -INFINITY, pl = 0.f;
  if (lane < n_splits) { pm = part_m[prow0 + (size_t)lane * 128]; pl = part_l[prow0 + (size_t)lane * 128]; }
  float po[ND][16];
  bf16x8 vv[ND][16];
#pragma unroll
  for (int u = 0; u < ND; ++u) {
    const int d = lane + 64 * u;
#pragma unroll
    for (int s = 0; s < 16; ++s) po[u][s] = s < n_splits ? part_o[(prow0 + (size_t)s * 128) * HD + d] : 0.f;
    const bf16_t* vr = vbT + (((size_t)c * Hkv + kvh) * HD + d) * Lp;
#pragma unroll
    for (int k = 0; k < 16; ++k) vv[u][k] = 8 * k < t8 ? *(const bf16x8*)(vr + 8 * k) : zero8;
  }

  // ---- scores of the candidate's own keys 0..t
#pragma unroll
  for (int u = 0; u < ND; ++u) qs[lane + 64 * u] = qv[u];
  sc[lane] = 0.f;
  sc[lane + 64] = 0.f;
  __syncthreads();
  float mx = pm;
  float dots[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    float dot = 0.f;
#pragma unroll
    for (int i8 = 0; i8 < HD / 8; ++i8)
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(qs[8 * i8 + e], (float)kv[kk][i8][e], dot);
    dots[kk] = lane + 64 * kk <= t ? dot * scale_log2e : -INFINITY;
    mx = fmaxf(mx, dots[kk]);
  }
  mx = ceilf(wave_max(mx));                     // finite (key t itself is always visible); an integer, so that
                                                // the bf16 rounding of the weights does not depend on the reference
  float l = 0.f;
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    float p = __builtin_amdgcn_exp2f(dots[kk] - mx);       // exp2(-inf) = 0 beyond t
    l += p;
    sc[lane + 64 * kk] = (float)(bf16_t)p;      // the weight that multiplies V is a bf16 operand
  }
  const float w = __builtin_amdgcn_exp2f(pm - mx);         // 0 for an empty split and for lanes >= n_splits
  if (lane < 16) wsplit[lane] = w;
  l += w * pl;
  l = wave_sum(l);
  __syncthreads();
  const float inv = 1.0f / l;
#pragma unroll
  for (int u = 0; u < ND; ++u) {
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) acc = fmaf(wsplit[s], po[u][s], acc);
#pragma unroll
    for (int k = 0; k < 16; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) {             // weights beyond t are 0; the values there may be anything
        const int jk = 8 * k + e;
        acc = fmaf(sc[jk], jk <= t ? (float)vv[u][k][e] : 0.f, acc);
      }
    out[((size_t)c * Hq + h) * HD + lane + 64 * u] = (bf16_t)(acc * inv);
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
  const bool fast = Lp <= 128 && n_splits <= 16;
  if (fast && md.hd == 128)
    attention_decode_merge_fast_kernel<128><<<dim3(g.B * g.n, md.Hq), 64, 0, s>>>(
        q, kb, vbT, part, part_m, part_l, out, g.n, md.Hq, md.Hkv, g.Lk, Lp, g.t0, q_tiles, n_splits, scale_log2e);
  else if (fast)
    attention_decode_merge_fast_kernel<64><<<dim3(g.B * g.n, md.Hq), 64, 0, s>>>(
        q, kb, vbT, part, part_m, part_l, out, g.n, md.Hq, md.Hkv, g.Lk, Lp, g.t0, q_tiles, n_splits, scale_log2e);
  else if (md.hd == 128)
    attention_decode_merge_kernel<128><<<dim3(g.B * g.n, md.Hq), 64, lds, s>>>(
        q, kb, vbT, part, part_m, part_l, out, g.n, md.Hq, md.Hkv, g.Lk, Lp, g.t0, q_tiles, n_splits, scale_log2e);
  else
    attention_decode_merge_kernel<64><<<dim3(g.B * g.n, md.Hq), 64, lds, s>>>(
        q, kb, vbT, part, part_m, part_l, out, g.n, md.Hq, md.Hkv, g.Lk, Lp, g.t0, q_tiles, n_splits, scale_log2e);
  return true;
}
