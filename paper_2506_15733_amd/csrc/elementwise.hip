// Bandwidth-bound glue kernels of the scoring pass: embedding gather, RMSNorm, rotary embedding,
// SiLU*mul, KV-page commit, PRM scalar head, log-softmax merge + block sum.
#include "common.h"

// ---------------------------------------------------------------- embedding
template <typename T>
__global__ void embed_kernel(const int32_t* __restrict__ tok, int tok_stride, const T* __restrict__ E,
                             float* __restrict__ x, int d, int V, int* status) {
  int m = blockIdx.x;
  int id = tok[(size_t)m * tok_stride];
  if (id < 0 || id >= V) {
    if (threadIdx.x == 0) report_status(status, SPECS_ETOKEN);
    id = id < 0 ? 0 : V - 1;
  }
  const T* row = E + (size_t)id * d;
  float* xo = x + (size_t)m * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) xo[c] = to_f32<T>(row[c]);
}
template <typename T>
void launch_embed(const int32_t* tok, int tok_stride, const T* E, float* x, int M, int d, int V, int* status,
                  hipStream_t s) {
  embed_kernel<T><<<M, 256, 0, s>>>(tok, tok_stride, E, x, d, V, status);
}
template void launch_embed<float>(const int32_t*, int, const float*, float*, int, int, int, int*, hipStream_t);
template void launch_embed<bf16_t>(const int32_t*, int, const bf16_t*, float*, int, int, int, int*, hipStream_t);

// ---------------------------------------------------------------- RMSNorm
// One 256-thread block per row. y = x * rsqrt(mean(x^2) + eps) * gain, float math, output in T.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return t;
}

template <typename T>
__device__ __forceinline__ void rmsnorm_row(const float* __restrict__ xr, const float* __restrict__ gain,
                                            T* __restrict__ yr, int d, float eps, float* red) {
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    float v = xr[c];
    ss += v * v;
  }
  ss = block_sum_256(ss, red);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += 256) yr[c] = from_f32<T>(xr[c] * inv * gain[c]);
}

// Vector form for rows of d <= 4096 floats, d % 4 == 0, 16-byte aligned: the row stays in registers (at most four
// float4 per thread) between the sum of squares and the scaled store. parts > 0: x (+)= sum of the K-split
// partial products P[parts][M][d] first (summed in slice order, then added to x), and x is written back.
template <typename T>
__device__ __forceinline__ void store4(T* p, float4 v);
template <>
__device__ __forceinline__ void store4<float>(float* p, float4 v) { *(float4*)p = v; }
template <>
__device__ __forceinline__ void store4<bf16_t>(bf16_t* p, float4 v) {
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 o = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
  *(bf16x4*)p = o;
}

template <int NW>
__device__ __forceinline__ float block_sum_waves(float v, float* red) {   // NW wavefronts, red[NW]
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += red[w];
  __syncthreads();
  return t;
}

// NT threads per row: 256 for many rows, 1024 for a few (one 16-byte column per thread, and the loads of the
// partial products of a column are issued four at a time so that their latencies overlap).
template <typename T, int NT>
__global__ void __launch_bounds__(NT) norm_rows_vec_kernel(float* __restrict__ x, const float* __restrict__ P,
                                                           int parts, int init, const float* __restrict__ gain,
                                                           T* __restrict__ out, size_t Md, int d, float eps) {
  constexpr int VPT = 1024 / NT;
  __shared__ float red[NT / 64];
  const size_t m = blockIdx.x;
  const int nv = d >> 2;
  float4* xr = (float4*)(x + m * d);
  float4 v[VPT];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    int c = threadIdx.x + i * NT;
    if (c < nv) {
      if (parts > 0) {
        const float4* pc = (const float4*)(P + m * d) + c;
        const size_t stride4 = Md >> 2;
        float4 acc = pc[0];
        for (int s0 = 1; s0 < parts; s0 += 4) {          // slices are added in order, loaded four at a time
          float4 q[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) q[k] = s0 + k < parts ? pc[(size_t)(s0 + k) * stride4] : float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int k = 0; k < 4; ++k) { acc.x += q[k].x; acc.y += q[k].y; acc.z += q[k].z; acc.w += q[k].w; }
        }
        if (!init) {
          float4 o = xr[c];
          acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
        }
        v[i] = acc;
        xr[c] = acc;
      } else {
        v[i] = xr[c];
      }
      ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    }
  }
  if (gain == nullptr) return;
  ss = block_sum_waves<NT / 64>(ss, red);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    int c = threadIdx.x + i * NT;
    if (c < nv) {
      float4 gn = ((const float4*)gain)[c];
      float4 y = {v[i].x * inv * gn.x, v[i].y * inv * gn.y, v[i].z * inv * gn.z, v[i].w * inv * gn.w};
      store4<T>(out + m * d + 4 * c, y);
    }
  }
}
template <typename T>
static void launch_norm_rows_vec(float* x, const float* P, int parts, int init, const float* gain, T* out, int M, int d,
                                 float eps, hipStream_t s) {
  if (M <= 64) norm_rows_vec_kernel<T, 1024><<<M, 1024, 0, s>>>(x, P, parts, init, gain, out, (size_t)M * d, d, eps);
  else norm_rows_vec_kernel<T, 256><<<M, 256, 0, s>>>(x, P, parts, init, gain, out, (size_t)M * d, d, eps);
}
static inline bool vec_rows_ok(int d, const void* a, const void* b, const void* c, const void* e) {
  return d % 4 == 0 && d <= 4096 && (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c | (uintptr_t)e) & 15) == 0;
}

template <typename T>
__global__ void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain, T* __restrict__ out, int d,
                               float eps) {
  __shared__ float red[4];
  size_t m = blockIdx.x;
  rmsnorm_row<T>(x + m * d, gain, out + m * d, d, eps, red);
}
template <typename T>
void launch_rmsnorm(const float* x, const float* gain, T* out, int M, int d, float eps, hipStream_t s) {
  if (vec_rows_ok(d, x, gain, out, nullptr))
    launch_norm_rows_vec<T>((float*)x, nullptr, 0, 0, gain, out, M, d, eps, s);
  else
    rmsnorm_kernel<T><<<M, 256, 0, s>>>(x, gain, out, d, eps);
}
template void launch_rmsnorm<float>(const float*, const float*, float*, int, int, float, hipStream_t);
template void launch_rmsnorm<bf16_t>(const float*, const float*, bf16_t*, int, int, float, hipStream_t);

// Consumer of a K-split projection: x (+)= sum of the partial products, then (optionally) the RMSNorm of the
// updated row, which the next projection reads. The partials are summed first, in slice order, and then added
// to the residual stream, so the result does not depend on how the workgroups were scheduled.
template <typename T>
__global__ void add_partials_rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ P, int parts, int init,
                                            const float* __restrict__ gain, T* __restrict__ out, size_t Md, int d,
                                            float eps) {
  __shared__ float red[4];
  size_t m = blockIdx.x;
  float* xr = x + m * d;
  const float* pr = P + m * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    float acc = pr[c];
    for (int sidx = 1; sidx < parts; ++sidx) acc += pr[sidx * Md + c];
    float v = init ? acc : xr[c] + acc;
    xr[c] = v;
    ss += v * v;
  }
  if (gain == nullptr) return;
  ss = block_sum_256(ss, red);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += 256) out[m * d + c] = from_f32<T>(xr[c] * inv * gain[c]);
}
template <typename T>
void launch_add_partials_rmsnorm(float* x, const float* P, int parts, int init, const float* gain, T* out, int M, int d,
                                 float eps, hipStream_t s) {
  if (vec_rows_ok(d, x, P, gain, out))
    launch_norm_rows_vec<T>(x, P, parts, init, gain, out, M, d, eps, s);
  else
    add_partials_rmsnorm_kernel<T><<<M, 256, 0, s>>>(x, P, parts, init, gain, out, (size_t)M * d, d, eps);
}
template void launch_add_partials_rmsnorm<float>(float*, const float*, int, int, const float*, float*, int, int, float,
                                                 hipStream_t);
template void launch_add_partials_rmsnorm<bf16_t>(float*, const float*, int, int, const float*, bf16_t*, int, int,
                                                  float, hipStream_t);

// Operand of the vocabulary head: the hidden state that PRECEDES each scored token.
template <typename T>
__global__ void rmsnorm_shifted_kernel(const float* __restrict__ x, const float* __restrict__ h_last,
                                       const float* __restrict__ gain, T* __restrict__ out, int nL, int L, int b0, int d,
                                       float eps) {
  __shared__ float red[4];
  size_t m = blockIdx.x;
  int b = (int)(m / nL), t = (int)(m % L);
  const float* src = (t == 0) ? h_last + (size_t)(b0 + b) * d : x + (m - 1) * d;
  rmsnorm_row<T>(src, gain, out + m * d, d, eps, red);
}
template <typename T>
void launch_rmsnorm_shifted(const float* x, const float* h_last, const float* gain, T* out, const BatchGeom& g, int d,
                            float eps, hipStream_t s) {
  rmsnorm_shifted_kernel<T><<<g.M, 256, 0, s>>>(x, h_last, gain, out, g.n * g.L, g.L, g.b0, d, eps);
}
template void launch_rmsnorm_shifted<float>(const float*, const float*, const float*, float*, const BatchGeom&, int,
                                            float, hipStream_t);
template void launch_rmsnorm_shifted<bf16_t>(const float*, const float*, const float*, bf16_t*, const BatchGeom&, int,
                                             float, hipStream_t);

// ---------------------------------------------------------------- rotary embedding
// cos/sin of pos * base^(-2i/hd), pos = context length + t, evaluated in double so that long
// contexts lose nothing; one table per call, shared by all layers and heads.
__global__ void rope_table_kernel(float* __restrict__ cs, int M, int nL, int L, int half, int hd, double base,
                                  const int32_t* __restrict__ lens, int b0, int len_override, int t0) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= M * half) return;
  int m = idx / half, i = idx % half;
  int b = m / nL, t = m % L;
  int ctx = len_override >= 0 ? len_override : lens[b0 + b];
  double ang = (double)(ctx + t0 + t) * pow(base, -2.0 * (double)i / (double)hd);
  double sn, cn;
  sincos(ang, &sn, &cn);
  cs[(size_t)m * hd + i] = (float)cn;
  cs[(size_t)m * hd + half + i] = (float)sn;
}
void launch_rope_table(float* cs, const BatchGeom& g, int hd, float base, hipStream_t s) {
  int half = hd / 2;
  int total = g.M * half;
  rope_table_kernel<<<(total + 255) / 256, 256, 0, s>>>(cs, g.M, g.n * g.L, g.L, half, hd, (double)base, g.lens, g.b0,
                                                        g.len_override, g.t0);
}

// qkv float [M, Hq+2Hkv, hd] -> q T [M,Hq,hd] (rotated), k T [cand*Lk + t][Hkv][hd] (rotated),
// v T transposed per candidate: vT[cand][Hkv][hd][Lp] (Lp = Lk rounded up to 16, padding zeroed), where row m is
// in-block position t = t0 + m % L of candidate m / L and Lk is the length of a whole block.
template <typename T>
__global__ void rope_split_kernel(const float* __restrict__ qkv, const float* __restrict__ cs, T* __restrict__ q,
                                  T* __restrict__ kblk, T* __restrict__ vT, int Hq, int Hkv, int hd, int Lrows, int t0,
                                  int L, int Lp, int parts, size_t part_stride) {
  size_t m = blockIdx.x;
  int H = Hq + 2 * Hkv, half = hd / 2;
  const float* in = qkv + m * (size_t)H * hd;
  const float* c = cs + m * hd;
  size_t cand = m / Lrows;
  int t = t0 + (int)(m % Lrows);
  const size_t krow = cand * L + t;
  // blockIdx.y strides over the heads (one block per row when gridDim.y == 1, one per (row, head) for few rows)
  const int heads_here = (H - (int)blockIdx.y + (int)gridDim.y - 1) / (int)gridDim.y;
  auto rotate = [&](int h, int i) {
    float x1 = in[h * hd + i], x2 = in[h * hd + half + i];
    for (int pidx = 1; pidx < parts; ++pidx) {           // K-split projection: add the slices up, in order
      x1 += in[pidx * part_stride + h * hd + i];
      x2 += in[pidx * part_stride + h * hd + half + i];
    }
    if (h < Hq + Hkv) {
      float cn = c[i], sn = c[half + i];
      float y1 = x1 * cn - x2 * sn, y2 = x2 * cn + x1 * sn;
      T* o = (h < Hq) ? q + (m * Hq + h) * hd : kblk + (krow * Hkv + (h - Hq)) * hd;
      o[i] = from_f32<T>(y1);
      o[half + i] = from_f32<T>(y2);
    } else {
      T* o = vT + ((cand * Hkv + (h - Hq - Hkv)) * hd) * Lp + t;
      o[(size_t)i * Lp] = from_f32<T>(x1);
      o[(size_t)(half + i) * Lp] = from_f32<T>(x2);
    }
  };
  if (blockDim.x % half == 0) {
    // thread -> (head slot, pair index) once, then whole head slots per pass: no division per element
    const int slots = blockDim.x / half, hs0 = threadIdx.x / half, i = threadIdx.x - hs0 * half;
    for (int hs = hs0; hs < heads_here; hs += slots) rotate(blockIdx.y + hs * gridDim.y, i);
  } else {
    for (int e = threadIdx.x; e < heads_here * half; e += blockDim.x)
      rotate(blockIdx.y + (e / half) * gridDim.y, e % half);
  }
  if (blockIdx.y == 0 && t == L - 1 && Lp > L) {
    for (int e = threadIdx.x; e < Hkv * hd; e += blockDim.x)
      for (int tt = L; tt < Lp; ++tt) vT[(cand * Hkv * hd + e) * Lp + tt] = from_f32<T>(0.f);
  }
}
template <typename T>
void launch_rope_split(const float* qkv, int parts, const float* cs, T* q, T* k, T* vT, const BatchGeom& g, int Lp,
                       const ModelDims& md, hipStream_t s) {
  size_t stride = (size_t)g.M * (md.Hq + 2 * md.Hkv) * md.hd;
  if (g.M <= 64)       // few rows: spread the heads over blocks of one wavefront
    rope_split_kernel<T><<<dim3(g.M, md.Hq + 2 * md.Hkv), 64, 0, s>>>(qkv, cs, q, k, vT, md.Hq, md.Hkv, md.hd, g.L, g.t0,
                                                                     g.Lk, Lp, parts, stride);
  else
    rope_split_kernel<T><<<g.M, 256, 0, s>>>(qkv, cs, q, k, vT, md.Hq, md.Hkv, md.hd, g.L, g.t0, g.Lk, Lp, parts, stride);
}
template void launch_rope_split<float>(const float*, int, const float*, float*, float*, float*, const BatchGeom&, int,
                                       const ModelDims&, hipStream_t);
template void launch_rope_split<bf16_t>(const float*, int, const float*, bf16_t*, bf16_t*, bf16_t*, const BatchGeom&,
                                        int, const ModelDims&, hipStream_t);

// v [M][Hkv][hd] -> vT [cand][Hkv][hd][Lp], zero padded (used when values arrive in token-major order)
template <typename T>
__global__ void transpose_v_kernel(const T* __restrict__ v, T* __restrict__ vT, int Hkv, int hd, int L, int Lp) {
  size_t cand = blockIdx.x;
  size_t per = (size_t)Hkv * hd;
  for (size_t e = threadIdx.x; e < per * Lp; e += blockDim.x) {
    size_t hc = e / Lp;
    int t = (int)(e % Lp);
    vT[cand * per * Lp + e] = t < L ? v[(cand * L + t) * per + hc] : from_f32<T>(0.f);
  }
}
template <typename T>
void launch_transpose_v(const T* v, T* vT, int cands, int Hkv, int hd, int L, int Lp, hipStream_t s) {
  transpose_v_kernel<T><<<cands, 256, 0, s>>>(v, vT, Hkv, hd, L, Lp);
}
template void launch_transpose_v<float>(const float*, float*, int, int, int, int, int, hipStream_t);
template void launch_transpose_v<bf16_t>(const bf16_t*, bf16_t*, int, int, int, int, int, hipStream_t);

// ---------------------------------------------------------------- SiLU(gate) * up
// gu float [M, 2F] in the interleaved-by-32 column order of the fused gate/up matrix.
template <typename T>
__global__ void silu_mul_kernel(const float* __restrict__ gu, T* __restrict__ act, int F) {
  size_t m = blockIdx.x;
  const float* in = gu + m * 2 * (size_t)F;
  for (int j = threadIdx.x; j < F; j += blockDim.x) {
    int col = (j / SPECS_GATE_UP_GROUP) * 2 * SPECS_GATE_UP_GROUP + (j % SPECS_GATE_UP_GROUP);
    float gte = in[col], up = in[col + SPECS_GATE_UP_GROUP];
    float sg = gte / (1.0f + expf(-gte));
    act[m * F + j] = from_f32<T>(sg * up);
  }
}
template <typename T>
void launch_silu_mul(const float* gu, T* act, int M, int F, hipStream_t s) {
  silu_mul_kernel<T><<<M, 256, 0, s>>>(gu, act, F);
}
template void launch_silu_mul<float>(const float*, float*, int, int, hipStream_t);
template void launch_silu_mul<bf16_t>(const float*, bf16_t*, int, int, hipStream_t);

// ---------------------------------------------------------------- KV commit into pages
// Copies the L block tokens of one candidate per beam (chosen[b], or candidate 0 when chosen == NULL)
// to positions ctx .. ctx+L-1 of the beam's pages: keys [page][Hkv][pt][hd], values transposed
// [page][Hkv][hd][pt]. grid = (L, B), one block per token.
template <typename T>
__global__ void kv_commit_kernel(const T* __restrict__ kb, const T* __restrict__ vbT, T* __restrict__ poolK,
                                 T* __restrict__ poolV, BatchGeom g, int Hkv, int hd, int Lp,
                                 const int32_t* __restrict__ chosen) {
  int t = blockIdx.x, b = blockIdx.y;
  int i = chosen ? chosen[b] : 0;
  i = i < 0 ? 0 : (i >= g.n ? g.n - 1 : i);          // an index a failed selection left (-1) must not address memory
  int ctx = g.len_override >= 0 ? g.len_override : g.lens[g.b0 + b];
  int pos = ctx + t;
  int page = g.page_table[(size_t)(g.b0 + b) * g.max_pages + pos / g.page_tokens];
  int slot = pos % g.page_tokens;
  size_t cand = (size_t)b * g.n + i;
  size_t m = cand * g.L + t;
  for (int e = threadIdx.x; e < Hkv * hd; e += blockDim.x) {
    int h = e / hd, c = e % hd;
    poolK[(((size_t)page * Hkv + h) * g.page_tokens + slot) * hd + c] = kb[m * Hkv * hd + e];
    poolV[(((size_t)page * Hkv + h) * hd + c) * g.page_tokens + slot] = vbT[(cand * Hkv * hd + e) * Lp + t];
  }
}
template <typename T>
void launch_kv_commit(const T* kb, const T* vbT, T* poolK, T* poolV, const BatchGeom& g, const ModelDims& md, int Lp,
                      const int32_t* chosen, hipStream_t s) {
  kv_commit_kernel<T><<<dim3(g.L, g.B), 256, 0, s>>>(kb, vbT, poolK, poolV, g, md.Hkv, md.hd, Lp, chosen);
}
template void launch_kv_commit<float>(const float*, const float*, float*, float*, const BatchGeom&, const ModelDims&,
                                      int, const int32_t*, hipStream_t);
template void launch_kv_commit<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, bf16_t*, const BatchGeom&,
                                       const ModelDims&, int, const int32_t*, hipStream_t);

// h_last[b0+b] = x[last row of candidate chosen[b] (or 0)]
__global__ void copy_rows_kernel(const float* __restrict__ x, float* __restrict__ h_last, BatchGeom g, int d,
                                 const int32_t* __restrict__ chosen) {
  int b = blockIdx.x;
  int i = chosen ? chosen[b] : 0;
  i = i < 0 ? 0 : (i >= g.n ? g.n - 1 : i);
  size_t m = ((size_t)b * g.n + i) * g.L + (g.L - 1);
  for (int c = threadIdx.x; c < d; c += blockDim.x) h_last[(size_t)(g.b0 + b) * d + c] = x[m * d + c];
}
void launch_copy_rows(const float* x, float* h_last, const BatchGeom& g, int d, const int32_t* chosen, hipStream_t s) {
  copy_rows_kernel<<<g.B, 256, 0, s>>>(x, h_last, g, d, chosen);
}

__global__ void broadcast_hlast_kernel(const float* __restrict__ h_last, float* __restrict__ xs, int n, int b0, int d) {
  size_t r = blockIdx.x;
  const float* src = h_last + (size_t)(b0 + r / n) * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) xs[r * d + c] = src[c];
}
void launch_broadcast_hlast(const float* h_last, float* xs, const BatchGeom& g, int d, hipStream_t s) {
  broadcast_hlast_kernel<<<g.B * g.n, 256, 0, s>>>(h_last, xs, g.n, g.b0, d);
}

template <typename T>
__global__ void gather_last_rows_kernel(const T* __restrict__ src, T* __restrict__ dst, int L, int width) {
  size_t c = blockIdx.x;
  for (int j = threadIdx.x; j < width; j += blockDim.x) dst[c * width + j] = src[(c * L + (L - 1)) * width + j];
}
template <typename T>
void launch_gather_last_rows(const T* src, T* dst, int C, int L, int width, hipStream_t s) {
  gather_last_rows_kernel<T><<<C, 256, 0, s>>>(src, dst, L, width);
}
template void launch_gather_last_rows<float>(const float*, float*, int, int, int, hipStream_t);
template void launch_gather_last_rows<bf16_t>(const bf16_t*, bf16_t*, int, int, int, hipStream_t);

__global__ void scatter_last_rows_kernel(const float* __restrict__ xs, float* __restrict__ x, int L, int d) {
  size_t c = blockIdx.x;
  for (int j = threadIdx.x; j < d; j += blockDim.x) x[(c * L + (L - 1)) * d + j] = xs[c * d + j];
}
void launch_scatter_last_rows(const float* xs, float* x, int C, int L, int d, hipStream_t s) {
  scatter_last_rows_kernel<<<C, 256, 0, s>>>(xs, x, L, d);
}

// ---------------------------------------------------------------- PRM scalar head
// r[b][i] = sigmoid(w_r . RMSNorm(x at the last block token)), all in float; one block per candidate.
template <typename T>
__global__ void prm_head_kernel(const float* __restrict__ x, const float* __restrict__ gain, const T* __restrict__ w,
                                float* __restrict__ out, int L, int d, float eps) {
  __shared__ float red[4];
  size_t c = blockIdx.x;
  const float* xr = x + (c * L + (L - 1)) * d;
  float ss = 0.f, dot = 0.f;
  for (int j = threadIdx.x; j < d; j += 256) {
    float v = xr[j];
    ss += v * v;
    dot += v * gain[j] * to_f32<T>(w[j]);
  }
  ss = block_sum_256(ss, red);
  dot = block_sum_256(dot, red);
  if (threadIdx.x == 0) {
    float sc = dot / sqrtf(ss / (float)d + eps);
    out[c] = 1.0f / (1.0f + expf(-sc));
  }
}
template <typename T>
void launch_prm_head(const float* x, const float* gain, const T* w, float* out, const BatchGeom& g, int d, float eps,
                     hipStream_t s) {
  prm_head_kernel<T><<<g.B * g.n, 256, 0, s>>>(x, gain, w, out, g.L, d, eps);
}
template void launch_prm_head<float>(const float*, const float*, const float*, float*, const BatchGeom&, int, float,
                                     hipStream_t);
template void launch_prm_head<bf16_t>(const float*, const float*, const bf16_t*, float*, const BatchGeom&, int, float,
                                      hipStream_t);

// ---------------------------------------------------------------- log-softmax merge + block sum
// Kernel 1, one wavefront per row: merge the per-tile (max, sum exp) partials,
// tok_logp = z[y] - (max + log sum). Kernel 2, one thread per candidate: add its L token terms in
// index order (fixed order => run-to-run identical), in double because the sum reaches ~1e3.
__global__ void lmhead_merge_kernel(const float* __restrict__ part_max, const float* __restrict__ part_sum,
                                    const float* __restrict__ zt, int n_tiles, float* __restrict__ tok_logp, int M) {
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  size_t m = (size_t)blockIdx.x * 4 + wave;
  if (m >= (size_t)M) return;
  const float* pm = part_max + m * n_tiles;
  const float* ps = part_sum + m * n_tiles;
  float mx = -INFINITY;
  for (int j = lane; j < n_tiles; j += 64) mx = fmaxf(mx, pm[j]);
  mx = wave_max(mx);
  float sm = 0.f;
  for (int j = lane; j < n_tiles; j += 64) sm += ps[j] * expf(pm[j] - mx);
  sm = wave_sum(sm);
  if (lane == 0) tok_logp[m] = (float)((double)zt[m] - ((double)mx + log((double)sm)));
}

__global__ void block_sum_kernel(const float* __restrict__ tok_logp, float* __restrict__ block_out, int L, int C) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  double acc = 0.0;
  for (int t = 0; t < L; ++t) acc += (double)tok_logp[(size_t)c * L + t];
  block_out[c] = (float)acc;
}

void launch_block_sum(const float* tok_logp, float* block_out, int L, int C, hipStream_t s) {
  block_sum_kernel<<<(C + 63) / 64, 64, 0, s>>>(tok_logp, block_out, L, C);
}

// tok_scratch: [M] floats used when the caller does not want the per-token terms
void launch_lmhead_merge(const float* part_max, const float* part_sum, const float* zt, int n_tiles, float* tok_logp,
                         float* tok_scratch, float* block_out, const BatchGeom& g, hipStream_t s) {
  float* tl = tok_logp ? tok_logp : tok_scratch;
  lmhead_merge_kernel<<<(g.M + 3) / 4, 256, 0, s>>>(part_max, part_sum, zt, n_tiles, tl, g.M);
  int C = g.B * g.n;
  block_sum_kernel<<<(C + 63) / 64, 64, 0, s>>>(tl, block_out, g.L, C);
}
