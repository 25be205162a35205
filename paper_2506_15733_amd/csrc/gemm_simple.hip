// Plain LDS-tiled SIMT GEMM, C = A[M,K] * W[N,K]^T with float accumulation, for the float
// configuration and for shapes the MFMA kernels do not take. Also the float version of the fused
// vocabulary head (per-tile log-sum-exp partials instead of logits).
#include "common.h"

#define TS 64   // tile of C per block
#define TK 16   // K step
// 256 threads, each a 4x4 patch of the 64x64 tile.

template <typename T>
__device__ __forceinline__ void load_tiles(const T* __restrict__ A, const T* __restrict__ W, int M, int N, int K,
                                           int m0, int n0, int k0, float (*As)[TS + 1], float (*Ws)[TS + 1]) {
  // 64 rows x 16 k = 1024 elements per operand, 4 per thread
  for (int e = threadIdx.x; e < TS * TK; e += 256) {
    int r = e / TK, kk = e % TK;
    int k = k0 + kk;
    float a = 0.f, w = 0.f;
    if (k < K) {
      if (m0 + r < M) a = to_f32<T>(A[(size_t)(m0 + r) * K + k]);
      if (n0 + r < N) w = to_f32<T>(W[(size_t)(n0 + r) * K + k]);
    }
    As[kk][r] = a;
    Ws[kk][r] = w;
  }
}

template <typename T>
__device__ __forceinline__ void tile_mainloop(const T* __restrict__ A, const T* __restrict__ W, int M, int N, int K,
                                              int m0, int n0, float acc[4][4]) {
  __shared__ float As[TK][TS + 1];
  __shared__ float Ws[TK][TS + 1];
  int tr = (threadIdx.x / 16) * 4, tc = (threadIdx.x % 16) * 4;
  for (int k0 = 0; k0 < K; k0 += TK) {
    load_tiles<T>(A, W, M, N, K, m0, n0, k0, As, Ws);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][tr + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tc + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
}

template <typename T, int EPI>
__global__ void __launch_bounds__(256) gemm_simple_kernel(const T* __restrict__ A, const T* __restrict__ W,
                                                          float* __restrict__ C, int M, int N, int K) {
  int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  float acc[4][4] = {};
  tile_mainloop<T>(A, W, M, N, K, m0, n0, acc);
  int tr = (threadIdx.x / 16) * 4, tc = (threadIdx.x % 16) * 4;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int m = m0 + tr + i, n = n0 + tc + j;
      if (m < M && n < N) {
        size_t o = (size_t)m * N + n;
        if (EPI == EPI_RESIDUAL_ADD) C[o] += acc[i][j];
        else C[o] = acc[i][j];
      }
    }
}

template <typename T>
void launch_gemm_simple(const T* A, const T* W, float* C, int M, int N, int K, GemmEpilogue epi, hipStream_t s) {
  dim3 grid((N + TS - 1) / TS, (M + TS - 1) / TS);
  if (epi == EPI_RESIDUAL_ADD) gemm_simple_kernel<T, EPI_RESIDUAL_ADD><<<grid, 256, 0, s>>>(A, W, C, M, N, K);
  else gemm_simple_kernel<T, EPI_STORE_F32><<<grid, 256, 0, s>>>(A, W, C, M, N, K);
}
template void launch_gemm_simple<float>(const float*, const float*, float*, int, int, int, GemmEpilogue, hipStream_t);
template void launch_gemm_simple<bf16_t>(const bf16_t*, const bf16_t*, float*, int, int, int, GemmEpilogue,
                                         hipStream_t);

// Vocabulary head without logits: each block reduces its 64 columns of every row to
// (max, sum exp(z - max)) and hands out z[target token] if the token falls in its columns.
template <typename T>
__global__ void __launch_bounds__(256) lmhead_partials_simple_kernel(const T* __restrict__ A, const T* __restrict__ W,
                                                                     const int32_t* __restrict__ tok,
                                                                     float* __restrict__ part_max,
                                                                     float* __restrict__ part_sum, float* __restrict__ zt,
                                                                     int M, int V, int K, int n_tiles) {
  int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  float acc[4][4] = {};
  tile_mainloop<T>(A, W, M, V, K, m0, n0, acc);
  int tr = (threadIdx.x / 16) * 4, tc = (threadIdx.x % 16) * 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + tr + i;
    int target = (m < M) ? tok[m] : -1;
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tc + j;
      if (n < V) mx = fmaxf(mx, acc[i][j]);
      if (n == target) zt[m] = acc[i][j];
    }
    // the 16 threads that share this row are 16 consecutive lanes
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float sm = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (n0 + tc + j < V) sm += expf(acc[i][j] - mx);
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) sm += __shfl_xor(sm, o, 64);
    if ((threadIdx.x % 16) == 0 && m < M) {
      part_max[(size_t)m * n_tiles + blockIdx.x] = mx;
      part_sum[(size_t)m * n_tiles + blockIdx.x] = sm;
    }
  }
}

int lmhead_simple_tiles(int V) { return (V + TS - 1) / TS; }

template <typename T>
void launch_lmhead_partials_simple(const T* A, const T* W, const int32_t* tok, float* part_max, float* part_sum,
                                   float* zt, int M, int V, int K, int* n_tiles_out, hipStream_t s) {
  int nt = lmhead_simple_tiles(V);
  dim3 grid(nt, (M + TS - 1) / TS);
  lmhead_partials_simple_kernel<T><<<grid, 256, 0, s>>>(A, W, tok, part_max, part_sum, zt, M, V, K, nt);
  *n_tiles_out = nt;
}
template void launch_lmhead_partials_simple<float>(const float*, const float*, const int32_t*, float*, float*, float*,
                                                   int, int, int, int*, hipStream_t);
template void launch_lmhead_partials_simple<bf16_t>(const bf16_t*, const bf16_t*, const int32_t*, float*, float*,
                                                    float*, int, int, int, int*, hipStream_t);
