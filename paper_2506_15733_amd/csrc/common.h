// Shared declarations of the HIP implementation (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "specs.h"

typedef __bf16 bf16_t;

// float <-> operand-type conversions. float -> bf16 is round-to-nearest-even (v_cvt_pk_bf16_f32).
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

// Device status word: the FIRST error since it was last cleared sticks (an ordinary global atomic compare-and-swap).
__device__ __forceinline__ void report_status(int* status, int code) { atomicCAS(status, 0, code); }

// Which implementation a launch took, counted per process (specs_path_counts): tests assert that the benchmark
// shapes run on the matrix-unit kernels and not on the plain ones that serve odd shapes.
void count_path(int which);

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// One scoring (or prefill-chunk) problem as the kernels see it.
// Row m of the activation matrices is token t of candidate i of beam b: m = (b*n + i)*L + t.
struct BatchGeom {
  int B, n, L;              // beams, candidates per beam, block tokens
  int M;                    // B*n*L
  int b0;                   // first beam of the prefix handle this launch covers (prefill: one beam at a time)
  int len_override;         // >= 0: context length used instead of lens[b] (prefill chunks)
  int t0;                   // in-block position of a row's first token: 0 when a launch covers whole blocks,
                            // t when it covers the single position t of every block (token-by-token generation)
  int Lk;                   // block length of the block key/value buffers (= L unless t0 > 0 launches are in use)
  const int32_t* lens;      // device [B_total]
  const int32_t* page_table;// device [B_total][max_pages]
  int max_pages, page_tokens;
};

struct ModelDims {
  int d, Hq, Hkv, hd, F, V;
  float eps, rope_base;
};

// ---- launchers implemented across the .hip files (all enqueue on `s`) ----
template <typename T>
void launch_embed(const int32_t* tok, int tok_stride, const T* E, float* x, int M, int d, int V, int* status,
                  hipStream_t s);   // row m embeds tok[m * tok_stride]
template <typename T>
void launch_rmsnorm(const float* x, const float* gain, T* out, int M, int d, float eps, hipStream_t s);
// lm_head operand: row (b,i,t) = norm(t == 0 ? h_last[b0+b] : x[row-1])
template <typename T>
void launch_rmsnorm_shifted(const float* x, const float* h_last, const float* gain, T* out, const BatchGeom& g,
                            int d, float eps, hipStream_t s);
void launch_rope_table(float* cs, const BatchGeom& g, int hd, float base, hipStream_t s);
// values leave this kernel transposed per candidate: vT[cand][Hkv][hd][Lp], Lp = L rounded up to 16
template <typename T>
void launch_rope_split(const float* qkv, int parts, const float* cs, T* q, T* k, T* vT, const BatchGeom& g, int Lp,
                       const ModelDims& md, hipStream_t s);   // qkv = sum of `parts` slices [M, (Hq+2Hkv)*hd]
template <typename T>
void launch_transpose_v(const T* v, T* vT, int cands, int Hkv, int hd, int L, int Lp, hipStream_t s);
template <typename T>
void launch_silu_mul(const float* gu, T* act, int M, int F, hipStream_t s);
template <typename T>
void launch_kv_commit(const T* kb, const T* vbT, T* poolK, T* poolV, const BatchGeom& g, const ModelDims& md,
                      int Lp, const int32_t* chosen, hipStream_t s);
template <typename T>
void launch_prm_head(const float* x, const float* gain, const T* w, float* out, const BatchGeom& g, int d, float eps,
                     hipStream_t s);
void launch_copy_rows(const float* x, float* h_last, const BatchGeom& g, int d, const int32_t* chosen, hipStream_t s);
// generation: xs[b*n + i] = h_last[b0 + b] (every candidate starts from the prefix's last hidden state)
void launch_broadcast_hlast(const float* h_last, float* xs, const BatchGeom& g, int d, hipStream_t s);
// dst[c][0..width) = src[(c*L + L-1)][0..width): the last row of every block
template <typename T>
void launch_gather_last_rows(const T* src, T* dst, int C, int L, int width, hipStream_t s);
// x[(c*L + L-1)] = xs[c] for every candidate c (the state at the last block token, where scoring leaves it)
void launch_scatter_last_rows(const float* xs, float* x, int C, int L, int d, hipStream_t s);
// block_out[c] = sum_t tok_logp[c][t] in index order, accumulated in double
void launch_block_sum(const float* tok_logp, float* block_out, int L, int C, hipStream_t s);
// Ancestral sampling of one token per row from softmax(logits[row, :limit]) by inverse CDF in id order from the
// uniform u[row*L + t]; writes the id to cand[row*L + t] and its log-probability to tok_logp[row*L + t].
// scratch: sample_scratch_bytes(rows) bytes, 8-byte aligned.
void launch_sample_tokens(const float* logits, int rows, int V, int limit, const double* u, int32_t* cand,
                          float* tok_logp, int L, int t, void* scratch, int* status, hipStream_t s);
size_t sample_scratch_bytes(int rows);

enum GemmEpilogue { EPI_STORE_F32 = 0, EPI_RESIDUAL_ADD = 1 };
// C[M,N] (float) = A[M,K] * W[N,K]^T, or C += ... (residual add)
template <typename T>
void launch_gemm_simple(const T* A, const T* W, float* C, int M, int N, int K, GemmEpilogue epi, hipStream_t s);

template <typename T>
void launch_attention_simple(const T* q, const T* kb, const T* vbT, const T* poolK, const T* poolV, T* out,
                             const BatchGeom& g, const ModelDims& md, int Lp, int max_ctx, hipStream_t s);
// part / part_floats: float scratch for launches that split the key tiles over workgroups (null: never split)
bool launch_attention_mfma(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* poolK,
                           const bf16_t* poolV, bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp,
                           int max_ctx, float* part, size_t part_floats, hipStream_t s);

// The same launches with the two-phase schedule (attention_pingpong.hip): 256 stacked rows of all candidates of a
// (beam, kv head) per workgroup. False if the shape is not taken.
bool launch_attention_pingpong(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* poolK,
                               const bf16_t* poolV, bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp,
                               int max_ctx, float* part, size_t part_floats, hipStream_t s);

// One in-block position per candidate (g.L == 1, position g.t0): prefix keys by the MFMA kernel in split mode,
// merged with the candidate's own block keys. part: scratch of part_floats floats. False if the shape is not taken.
bool launch_attention_decode(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* poolK,
                             const bf16_t* poolV, bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp,
                             int max_ctx, float* part, size_t part_floats, hipStream_t s);

// Fused vocabulary head: per (row, 64-column tile) partial (max, sum exp) and the target-token logit.
template <typename T>
void launch_lmhead_partials_simple(const T* A, const T* W, const int32_t* tok, float* part_max, float* part_sum,
                                   float* zt, int M, int V, int K, int* n_tiles_out, hipStream_t s);
int lmhead_simple_tiles(int V);
void launch_lmhead_merge(const float* part_max, const float* part_sum, const float* zt, int n_tiles, float* tok_logp,
                         float* tok_scratch, float* block_out, const BatchGeom& g, hipStream_t s);

// gen_is_draft (device [B], in/out; requires nb == 1) / tau: Alg. 1 Steps II-III in one launch: beams whose flag is 0
// take pi_gen = pi_target (lg is ignored for them), and after the selection a beam with max_i r > tau sets its flag.
void launch_subsample(const float* lt, const float* lg, const float* r, const uint8_t* mask, int B, int n,
                      const float* beta_dev, int nb, const double* u, int32_t* idx, float* max_reward,
                      uint8_t* gen_is_draft, float tau, int* status, hipStream_t s);

// bf16 MFMA GEMM family (gemm_mfma.hip). Returns false if the shape is not supported.
enum { MFMA_STORE = 0, MFMA_RESIDUAL = 1, MFMA_SWIGLU = 2, MFMA_LMHEAD = 3 };
// ksplit > 1 (MFMA_STORE only): C is [ksplit][M][N], one partial product per K slice; bm = 128, 256 or 0 (auto).
bool launch_gemm_mfma(int epi, const bf16_t* A, const bf16_t* W, int M, int N, int K, float* C, bf16_t* act,
                      const int32_t* tok, float* part_max, float* part_sum, float* zt, int ksplit, int bm,
                      hipStream_t s);
bool launch_gemm_mfma_qkv_rope(const bf16_t* A, const bf16_t* W, const float* cs, bf16_t* q, bf16_t* kblk, bf16_t* vT,
                               const BatchGeom& g, const ModelDims& md, int Lp, hipStream_t s);
// tile height and number of K slices for a product whose consumer sums up to max_split partial products
void mfma_gemm_plan(int M, int N, int K, int max_split, int* bm_out, int* split_out);
// x[M,d] (+)= sum of `parts` partial products P[parts][M,d]; init != 0 overwrites x instead of adding to it.
// With gain != nullptr also out = RMSNorm(x) * gain (the operand of the next projection).
template <typename T>
void launch_add_partials_rmsnorm(float* x, const float* P, int parts, int init, const float* gain, T* out, int M, int d,
                                 float eps, hipStream_t s);
int mfma_lmhead_tiles(int V);
// Weight-streaming GEMM for M <= 32 rows (gemm_skinny.hip): MFMA_STORE writes ksplit partial products
// [ksplit][M][N]; MFMA_SWIGLU (ksplit 1) writes silu(gate)*up. Returns false if the shape is not taken.
bool launch_gemm_skinny(int epi, const bf16_t* A, const bf16_t* W, int M, int N, int K, float* C, bf16_t* act,
                        int ksplit, hipStream_t s);
int skinny_gemm_split(int N, int K, int max_split);
