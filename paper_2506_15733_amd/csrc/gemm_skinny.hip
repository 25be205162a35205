// Weight-streaming GEMM for at most 32 activation rows (token-by-token generation): C[M,N] = A[M,K] * W[N,K]^T,
// bf16 operands, float accumulation, K % 128 == 0. Every weight byte is read once and used for M <= 32
// multiply-adds, so the kernel is bound by HBM bandwidth and is organised around keeping loads in flight:
//   * a wavefront owns 16 weight rows and walks along K in slabs of 128: four 16-byte loads per lane per slab
//     straight into registers (64 contiguous bytes per row and instruction), the next slab (the next three, when a
//     launch has only a few wavefronts per CU) requested before the current one is multiplied;
//   * the weight rows are the A operand of v_mfma_f32_16x16x32_bf16, the (few) activation rows its B operand,
//     read from an LDS copy of A that the workgroup's four or eight wavefronts share (staged 1024 columns at a time,
//     16-byte chunks XOR-swizzled by the token index so that the 16 tokens of a read hit distinct banks);
//   * K is cut into gridDim.y slices so that short N still yields a few thousand wavefronts; slice s writes its
//     partial product to C + s*M*N and the consumer adds the slices up.
// Epilogues: float store (partial products, or the result itself with one slice), or SwiGLU: the wavefront's 16
// rows are then the gate rows and the up rows of the same 8 units (the fused gate/up matrix interleaves them in
// groups of 32 rows) and it writes silu(gate) * up as bf16.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

enum { SK_STORE = 0, SK_SWIGLU = 1 };

struct SkinnyArgs {
  const bf16_t* A;   // [M][K]
  const bf16_t* W;   // [N][K]
  float* C;          // SK_STORE: [ksplit][M][N]
  bf16_t* act;       // SK_SWIGLU: [M][N/2]
  int M, N, K, ksplit;
};

template <int TG, int EPI, int WPB, int PF>
__global__ void __launch_bounds__(64 * WPB) gemm_skinny_kernel(SkinnyArgs a) {
  constexpr int STAGE_COLS = 1024;                       // activation columns resident in LDS
  constexpr int ROWB = STAGE_COLS * 2;                   // bytes per LDS row
  constexpr int NSUB = 1;                                // weight-row sets per wavefront
  __shared__ __attribute__((aligned(16))) char As[16 * TG * ROWB];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, c = lane >> 4;
  const int wt = blockIdx.x * WPB + wave;                  // 16-row (SwiGLU: 16-unit) tile of this wavefront
  int wrow[NSUB];
  bool live;
  if (EPI == SK_SWIGLU) {
    // A-operand rows 0..7: the gate rows of units 8*wt .. 8*wt+7, rows 8..15: their up rows (the fused matrix keeps
    // the gate rows of units 32Q..32Q+31 at 64Q.., their up rows 32 further)
    const int unit = 8 * wt + (r & 7);
    wrow[0] = 64 * (unit >> 5) + (unit & 31) + (r >> 3) * 32;
    live = 16 * wt < a.N;
  } else {
    wrow[0] = wt * 16 + r;
    live = wt * 16 < a.N;
  }
  const bf16_t* wp[NSUB];
#pragma unroll
  for (int u = 0; u < NSUB; ++u) {
    int row = wrow[u] < a.N ? wrow[u] : a.N - 1;         // rows past the end are loaded from the last row, never stored
    wp[u] = a.W + (size_t)row * a.K + 8 * c;
  }
  const int KT = a.K >> 7;                               // slabs of 128 columns
  const int kt0 = (int)((long)blockIdx.y * KT / a.ksplit), kt1 = (int)((long)(blockIdx.y + 1) * KT / a.ksplit);

  floatx4 acc[NSUB][TG];
#pragma unroll
  for (int u = 0; u < NSUB; ++u)
#pragma unroll
    for (int g = 0; g < TG; ++g) acc[u][g] = floatx4{0.f, 0.f, 0.f, 0.f};

  // PF register sets take turns: while one slab is multiplied the loads of the next PF-1 are in flight, which is
  // what keeps HBM busy when a launch has only a few wavefronts per CU
  static_assert((STAGE_COLS / 128) % PF == 0, "a stage must hold a whole number of register-set rounds");
  bf16x8 w[PF][NSUB][4];
  auto load_slab = [&](int kt, bf16x8 (&dst)[NSUB][4]) {
    if (kt >= kt1) return;                               // past the end of the slice: nothing to fetch
#pragma unroll
    for (int u = 0; u < NSUB; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) dst[u][j] = *(const bf16x8*)(wp[u] + (size_t)kt * 128 + 32 * j);
  };
  auto multiply = [&](int slab_in_stage, const bf16x8 (&w)[NSUB][4]) {
    const int chbase = slab_in_stage * 16 + c;           // chunk of this lane's k-offset 8c within the slab, + 4j below
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int g = 0; g < TG; ++g) {
        const int m = g * 16 + r;
        bf16x8 bv = *(const bf16x8*)(As + m * ROWB + (((chbase + 4 * j) ^ r) << 4));
#pragma unroll
        for (int u = 0; u < NSUB; ++u)
          acc[u][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[u][j], bv, acc[u][g], 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int i = 0; i < PF - 1; ++i) load_slab(kt0 + i, w[i]);
  int kt = kt0, s0 = kt0;
  while (kt < kt1) {
    if (((kt - kt0) & (STAGE_COLS / 128 - 1)) == 0) {
      s0 = kt;
      const int s1 = s0 + STAGE_COLS / 128 < kt1 ? s0 + STAGE_COLS / 128 : kt1;
      __syncthreads();                                   // everybody is done with the previous stage
      // stage A[:, s0*128 .. s1*128): 16-byte chunk ch of token row m goes to chunk position ch ^ (m & 15)
      const int chunks_per_row = (s1 - s0) * 16;
      for (int q = tid; q < 16 * TG * chunks_per_row; q += 64 * WPB) {
        int m = q / chunks_per_row, ch = q - m * chunks_per_row;
        bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (m < a.M) v = *(const bf16x8*)(a.A + (size_t)m * a.K + (size_t)s0 * 128 + ch * 8);
        *(bf16x8*)(As + m * ROWB + ((ch ^ (m & 15)) << 4)) = v;
      }
      __syncthreads();
    }
    // one round: slab kt + i is in set i; set (i + PF - 1) % PF is refilled with slab kt + i + PF - 1
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      if (kt + i < kt1) {
        load_slab(kt + i + PF - 1, w[(i + PF - 1) % PF]);
        multiply(kt + i - s0, w[i]);
      }
    }
    kt += PF;
  }
  if (!live) return;
  // accumulator element e of this lane: weight row 4c + e of the tile, token r (+ 16 per token group)
  if (EPI == SK_STORE) {
    float* Cs = a.C + (size_t)blockIdx.y * a.M * a.N;
    const int n = wt * 16 + 4 * c;
#pragma unroll
    for (int g = 0; g < TG; ++g) {
      const int m = g * 16 + r;
      if (m >= a.M) continue;
      float* dst = Cs + (size_t)m * a.N + n;
      if (n + 3 < a.N && (a.N & 3) == 0) {
        *(float4*)dst = float4{acc[0][g][0], acc[0][g][1], acc[0][g][2], acc[0][g][3]};
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < a.N) dst[e] = acc[0][g][e];
      }
    }
  } else {
    // lanes c = 0, 1 hold the gate values of units 4c + e, lanes c = 2, 3 (32 lanes further) the up values of the same
    // units: one exchange across the half-wave pairs them
    const int F = a.N >> 1;
    const int unit = 8 * wt + 4 * (c & 1);
#pragma unroll
    for (int g = 0; g < TG; ++g) {
      const int m = g * 16 + r;
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float mine = acc[0][g][e];
        float other = __shfl_xor(mine, 32, 64);
        float gt = c < 2 ? mine : other, up = c < 2 ? other : mine;
        o[e] = (__bf16)(gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * up);
      }
      if (c < 2 && m < a.M) *(bf16x4*)(a.act + (size_t)m * F + unit) = o;
    }
  }
}

// Number of K slices for an M x N x K product with M <= 32: enough wavefronts to keep every CU's load queues
// full (about 2048), at least four slabs of 128 columns per slice, at most max_split slices.
int skinny_gemm_split(int N, int K, int max_split) {
  int KT = K / 128;
  int want = (2048 * 16 + N - 1) / N;
  int cap = KT / 4 > 0 ? KT / 4 : 1;
  int sp = want < cap ? want : cap;
  sp = sp < max_split ? sp : max_split;
  return sp < 1 ? 1 : sp;
}

// epi: MFMA_STORE (C = [ksplit][M][N] partial products) or MFMA_SWIGLU (act, ksplit must be 1).
// Returns false if the shape is not taken.
bool launch_gemm_skinny(int epi, const bf16_t* A, const bf16_t* W, int M, int N, int K, float* C, bf16_t* act,
                        int ksplit, hipStream_t s) {
  if (M <= 0 || M > 32 || K % 128 != 0 || N <= 0 || ksplit < 1 || ksplit > K / 128) return false;
  if (((uintptr_t)A | (uintptr_t)W) & 15) return false;
  if (epi == MFMA_SWIGLU && (N % 64 != 0 || ksplit != 1 || ((uintptr_t)act & 7))) return false;
  if (epi != MFMA_SWIGLU && epi != MFMA_STORE) return false;
  if (epi == MFMA_STORE && ((uintptr_t)C & 15)) return false;
  SkinnyArgs a;
  a.A = A; a.W = W; a.C = C; a.act = act; a.M = M; a.N = N; a.K = K; a.ksplit = ksplit;
  int tiles = (N + 15) / 16;                                     // wavefront tiles (SwiGLU: 8 units = 16 rows each)
  // eight wavefronts share one LDS copy of A where that still leaves two workgroups per CU, else four
  bool wide = (long)((tiles + 7) / 8) * ksplit >= 512;
  dim3 grid(wide ? (tiles + 7) / 8 : (tiles + 3) / 4, ksplit);
  // few wavefronts per CU: three slabs in flight per wavefront instead of one
  const bool deep = (long)grid.x * grid.y * (wide ? 8 : 4) < 256 * 8;
#define SKINNY(TG, E)                                                                  \
  if (wide) gemm_skinny_kernel<TG, E, 8, 2><<<grid, 512, 0, s>>>(a);                   \
  else if (deep) gemm_skinny_kernel<TG, E, 4, 4><<<grid, 256, 0, s>>>(a);              \
  else gemm_skinny_kernel<TG, E, 4, 2><<<grid, 256, 0, s>>>(a)
  if (epi == MFMA_SWIGLU) {
    if (M <= 16) { SKINNY(1, SK_SWIGLU); } else { SKINNY(2, SK_SWIGLU); }
  } else {
    if (M <= 16) { SKINNY(1, SK_STORE); } else { SKINNY(2, SK_STORE); }
  }
#undef SKINNY
  return true;
}
