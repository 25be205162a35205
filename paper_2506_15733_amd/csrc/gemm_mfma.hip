// bf16 MFMA GEMM for gfx950: C[M,N] = A[M,K] * W[N,K]^T, float accumulation, K % 64 == 0.
//
// Block tile BM x 256 x 64 (BM = 256 or 128), 512 threads = 8 wavefronts laid out 2 (M) x 4 (N);
// every wavefront owns a (BM/2) x 64 patch as (BM/64) x 2 accumulators of
// v_mfma_f32_32x32x16_bf16. Operand tiles go global -> LDS directly (16 bytes per lane,
// no register staging), double buffered: the loads of K-tile t+1 are in flight while K-tile t
// is multiplied. LDS rows are 128 bytes (64 bf16); the 16-byte chunk c of row r is stored at
// chunk position c ^ ((r >> 1) & 7) so that the 32 rows a fragment read touches spread over all
// banks. Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id -> tile map
// below keeps all M-tiles of one N-tile on one XCD, so a weight tile is fetched from HBM once
// and re-used out of that XCD's L2.
//
// Epilogues: plain float store; residual add into the float stream; SwiGLU (gate/up columns
// interleaved in groups of 32 so that a lane holds gate and up of the same unit) with bf16
// output; vocabulary head: per-row (max, sum exp) over the tile's 256 columns plus the logit of
// the row's target token, so that logits never reach memory.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

enum MfmaEpilogue { ME_STORE = 0, ME_RESIDUAL = 1, ME_SWIGLU = 2, ME_LMHEAD = 3 };

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* W;
  int M, N, K;
  int m_tiles, n_tiles;
  float* C;              // ME_STORE / ME_RESIDUAL: [M, N]
  bf16_t* act;           // ME_SWIGLU: [M, N/2]
  const int32_t* tok;    // ME_LMHEAD: target token per row
  float* part_max;       // ME_LMHEAD: [M, n_tiles]
  float* part_sum;
  float* zt;             // ME_LMHEAD: [M]
};

// One direct-to-LDS load instruction: span p (8 wavefronts x 1 KiB = 64 rows of 128 bytes) of an operand tile.
__device__ __forceinline__ void load_span_async(const bf16_t* __restrict__ G, int row0, int rows_total, int K, int k0,
                                                char* lds_tile, int p) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int span = p * 8 + wave;                   // 1 KiB of LDS = 8 rows, written by one wavefront
  int q = span * 64 + lane;
  int row = q >> 3, slot = q & 7;
  int chunk = slot ^ ((row >> 1) & 7);
  int grow = row0 + row;
  grow = grow < rows_total ? grow : rows_total - 1;
  const bf16_t* src = G + (size_t)grow * K + k0 + chunk * 8;
  __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(lds_tile + span * 1024), 16, 0, 0);
}

__device__ __forceinline__ bf16x8 lds_frag(const char* tile, int row, int chunk) {
  return *(const bf16x8*)(tile + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
}

template <int BM, int EPI>
__global__ void __launch_bounds__(512) gemm_mfma_kernel(GemmArgs a) {
  constexpr int BN = 256;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  constexpr int WM = BM / 2, TM = WM / 32, TN = 2;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // id -> (m_tile, n_tile): ids congruent mod 8 share an XCD; consecutive ids there walk the M-tiles of one N-tile
  const int id = blockIdx.x;
  const int xcd = id & 7, seq = id >> 3;
  const int m_tile = seq % a.m_tiles;
  const int n_tile = (seq / a.m_tiles) * 8 + xcd;
  if (n_tile >= a.n_tiles) return;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 2, wn = wave & 3;
  const int lrow = lane & 31, lhalf = lane >> 5;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = a.K / 64;
  auto read_frags = [&](const char* As, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
    const char* Bs = As + A_BYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = lds_frag(As, wm * WM + i * 32 + lrow, ks * 2 + lhalf);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = lds_frag(Bs, wn * 64 + j * 32 + lrow, ks * 2 + lhalf);
  };
  auto mma = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };
  constexpr int LA = BM / 64, LB = BN / 64, LPT = LA + LB;   // direct-to-LDS loads per thread per K-tile
  // load instruction i (0 .. LPT-1) of K-tile t into ring buffer `buf`
  auto issue = [&](int i, int t, char* buf) {
    if (i < LA) load_span_async(a.A, m0, a.M, a.K, t * 64, buf, i);
    else load_span_async(a.W, n0, a.N, a.K, t * 64, buf + A_BYTES, i - LA);
  };
  // One k-step of the software pipeline: two MFMAs of the current group go first, then the LDS reads of the
  // next group (and, in the first k-step, the next K-tile's global loads) are issued, then the rest of the
  // MFMAs. Nothing in the group waits on those reads.
#define PIPE_STEP_ORDER(NLOADS)                                        \
  __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                   \
  __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);             \
  __builtin_amdgcn_sched_group_barrier(0x010, NLOADS, 0);              \
  __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - 2, 0);         \
  __builtin_amdgcn_sched_barrier(0)

  constexpr int L0 = LPT, L1 = 0, L2 = 0;

#pragma unroll
  for (int i = 0; i < LPT; ++i) issue(i, 0, smem);
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
  read_frags(smem, 0, a0, b0);
  for (int kt = 0; kt < KT; ++kt) {
    const char* cur = smem + (kt & 1) * STAGE;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    // The loop body is branch-free so that each k-step stays one scheduling region: on the last K-tile the
    // "next" tile is the last one again (a redundant reload into the free buffer, never consumed).
    const int tn = kt + 1 < KT ? kt + 1 : KT - 1;
    // every wavefront is past the barrier that ended K-tile kt-1, so its buffer (nxt) is free
    read_frags(cur, 1, a1, b1);
#pragma unroll
    for (int i = 0; i < L0; ++i) issue(i, tn, nxt);
    mma(a0, b0);
    PIPE_STEP_ORDER(L0);
    read_frags(cur, 2, a0, b0);
#pragma unroll
    for (int i = L0; i < L0 + L1; ++i) issue(i, tn, nxt);
    mma(a1, b1);
    PIPE_STEP_ORDER(L1);
    read_frags(cur, 3, a1, b1);
#pragma unroll
    for (int i = L0 + L1; i < LPT; ++i) issue(i, tn, nxt);
    mma(a0, b0);
    PIPE_STEP_ORDER(L2);
    // publish K-tile kt+1: own loads landed, own reads of K-tile kt complete, then meet the other wavefronts
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    read_frags(nxt, 0, a0, b0);
    mma(a1, b1);
    PIPE_STEP_ORDER(0);
  }
#undef PIPE_STEP_ORDER

  // accumulator element r of lane: row 8*(r/4) + 4*lhalf + r%4, column lrow of the 32x32 tile
  if (EPI == ME_STORE || EPI == ME_RESIDUAL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int col = n0 + wn * 64 + j * 32 + lrow;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int row = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
          if (row < a.M && col < a.N) {
            size_t o = (size_t)row * a.N + col;
            if (EPI == ME_RESIDUAL) a.C[o] += acc[i][j][r];
            else a.C[o] = acc[i][j][r];
          }
        }
      }
  } else if (EPI == ME_SWIGLU) {
    const int F = a.N >> 1;
    int fcol = ((n0 + wn * 64) >> 1) + lrow;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int row = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        float g = acc[i][0][r], u = acc[i][1][r];
        float v = g / (1.0f + expf(-g)) * u;
        if (row < a.M && fcol < F) a.act[(size_t)row * F + fcol] = (bf16_t)v;
      }
  } else {  // ME_LMHEAD
    __syncthreads();                                   // every wavefront is done with the operand tiles
    float* red_max = (float*)smem;                     // [BM][4]
    float* red_sum = red_max + BM * 4;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int lr = wm * WM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        int row = m0 + lr;
        int target = row < a.M ? a.tok[row] : -1;
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          int col = n0 + wn * 64 + j * 32 + lrow;
          if (col < a.N) mx = fmaxf(mx, acc[i][j][r]);
          if (col == target) a.zt[row] = acc[i][j][r];
        }
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        float sm = 0.f;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          int col = n0 + wn * 64 + j * 32 + lrow;
          if (col < a.N) sm += expf(acc[i][j][r] - mx);
        }
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) sm += __shfl_xor(sm, o, 64);
        if (lrow == 0) {
          red_max[lr * 4 + wn] = mx;
          red_sum[lr * 4 + wn] = sm;
        }
      }
    __syncthreads();
    for (int lr = threadIdx.x; lr < BM; lr += 512) {
      int row = m0 + lr;
      if (row < a.M) {
        float mx = fmaxf(fmaxf(red_max[lr * 4], red_max[lr * 4 + 1]), fmaxf(red_max[lr * 4 + 2], red_max[lr * 4 + 3]));
        float sm = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w)
          if (red_max[lr * 4 + w] > -INFINITY) sm += red_sum[lr * 4 + w] * expf(red_max[lr * 4 + w] - mx);
        a.part_max[(size_t)row * a.n_tiles + n_tile] = mx;
        a.part_sum[(size_t)row * a.n_tiles + n_tile] = sm;
      }
    }
  }
}

template <int BM, int EPI>
static void launch_variant(const GemmArgs& a, hipStream_t s) {
  constexpr int smem = 2 * (BM * 128 + 256 * 128);
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    configured = true;
  }
  int groups = (a.n_tiles + 7) / 8;
  gemm_mfma_kernel<BM, EPI><<<dim3(groups * 8 * a.m_tiles), 512, smem, s>>>(a);
}

int mfma_lmhead_tiles(int V) { return (V + 255) / 256; }

// Returns false when the shape is not one this kernel takes (the caller then uses the SIMT kernel).
bool launch_gemm_mfma(int epi, const bf16_t* A, const bf16_t* W, int M, int N, int K, float* C, bf16_t* act,
                      const int32_t* tok, float* part_max, float* part_sum, float* zt, hipStream_t s) {
  if (K % 64 != 0 || M <= 0 || N <= 0) return false;
  if (epi == ME_SWIGLU && (N % 64 != 0)) return false;
  GemmArgs a;
  a.A = A; a.W = W; a.M = M; a.N = N; a.K = K; a.C = C; a.act = act; a.tok = tok;
  a.part_max = part_max; a.part_sum = part_sum; a.zt = zt;
  a.n_tiles = (N + 255) / 256;
  // 128-row tiles when 256-row tiles would leave most of the 256 CUs idle
  bool small = ((M + 255) / 256) * a.n_tiles < 200 || M <= 128;
  a.m_tiles = small ? (M + 127) / 128 : (M + 255) / 256;
#define DISPATCH(E)                                   \
  if (small) launch_variant<128, E>(a, s);            \
  else launch_variant<256, E>(a, s);
  switch (epi) {
    case ME_STORE: DISPATCH(ME_STORE); break;
    case ME_RESIDUAL: DISPATCH(ME_RESIDUAL); break;
    case ME_SWIGLU: DISPATCH(ME_SWIGLU); break;
    case ME_LMHEAD: DISPATCH(ME_LMHEAD); break;
    default: return false;
  }
#undef DISPATCH
  return true;
}
