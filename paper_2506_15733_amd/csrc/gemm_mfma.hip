// bf16 MFMA GEMM for gfx950: C[M,N] = A[M,K] * W[N,K]^T, float accumulation, K % 64 == 0.
//
// Block tile BM x 256 x 64 (BM = 256 or 128), 512 threads = 8 wavefronts laid out 2 (M) x 4 (N);
// every wavefront owns a (BM/2) x 64 patch as (BM/64) x 2 accumulators of
// v_mfma_f32_32x32x16_bf16. Operand tiles go global -> LDS directly (16 bytes per lane,
// no register staging) into a ring of five 32 KiB slots: two being multiplied, three in flight.
// Wavefronts issue in order and the vector-memory queue is short, so the eight loads a wavefront
// contributes per k-step are dealt over the k-step's four MFMA groups, one load between MFMAs,
// instead of one burst; the k-loop is unrolled by the ring length so that slot addresses are
// constants. LDS rows are 128 bytes (64 bf16); the 16-byte chunk c of row r is stored at
// chunk position c ^ ((r >> 1) & 7) so that the 32 rows a fragment read touches spread over all
// banks. Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id -> tile map
// below keeps all M-tiles of one N-tile on one XCD, so a weight tile is fetched from HBM once
// and re-used out of that XCD's L2 by workgroups that walk through K in step.
//
// Epilogues: plain float store; residual add into the float stream; SwiGLU (gate/up columns
// interleaved in groups of 32 so that a lane holds gate and up of the same unit) with bf16
// output; vocabulary head: per-row (max, sum exp) over the tile's 256 columns plus the logit of
// the row's target token, so that logits never reach memory.
#include "common.h"
#include <type_traits>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

enum MfmaEpilogue { ME_STORE = 0, ME_RESIDUAL = 1, ME_SWIGLU = 2, ME_LMHEAD = 3, ME_QKV_ROPE = 4 };

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* W;
  int M, N, K;
  int m_tiles, n_tiles;
  int m_blocks;          // ceil(m_tiles / 8)
  float* C;              // ME_STORE / ME_RESIDUAL: [M, N]
  bf16_t* act;           // ME_SWIGLU: [M, N/2]
  const int32_t* tok;    // ME_LMHEAD: target token per row
  float* part_max;       // ME_LMHEAD: [M, n_tiles]
  float* part_sum;
  float* zt;             // ME_LMHEAD: [M]
  int ksplit;            // ME_STORE only: gridDim.y slices of K, slice s writes its partial product to C + s*M*N
  // ME_QKV_ROPE: the product is the QKV projection [M, (Hq + 2 Hkv) * hd]; the epilogue rotates the q and k heads
  // (pairs (i, i + hd/2), angles from the table cs[M][hd] = cos | sin) and writes bf16 q [M][Hq][hd], block keys
  // kblk[cand*Lk + t][Hkv][hd] and block values transposed per candidate vT[cand][Hkv][hd][Lp], where row m is
  // in-block position t = t0 + m % Lrows of candidate m / Lrows.
  const float* cs;
  bf16_t* q;
  bf16_t* kblk;
  bf16_t* vT;
  int Hq, Hkv, hd, Lrows, t0, Lk, Lp;
};

// One direct-to-LDS load instruction: the workgroup's NW wavefronts write NW consecutive 1 KiB spans
// (8 rows of 128 bytes each) of an operand tile.
// SWAP56: LDS row r holds tile row r with bits 5 and 6 exchanged (see the ME_QKV_ROPE epilogue).
template <int NW, bool SWAP56 = false>
__device__ __forceinline__ void load_span_async(const bf16_t* __restrict__ G, int row0, int rows_total, int K, int k0,
                                                char* lds_tile, int p, int wave) {
  const int lane = threadIdx.x & 63;
  int span = p * NW + wave;                  // 1 KiB of LDS = 8 rows, written by one wavefront
  int q = span * 64 + lane;
  int row = q >> 3, slot = q & 7;
  int chunk = slot ^ ((row >> 1) & 7);
  int grow = row0 + (SWAP56 ? ((row & ~0x60) | ((row & 0x20) << 1) | ((row & 0x40) >> 1)) : row);
  grow = grow < rows_total ? grow : rows_total - 1;
  const bf16_t* src = G + (size_t)grow * K + k0 + chunk * 8;
  __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(lds_tile + span * 1024), 16, 0, 0);
}

__device__ __forceinline__ bf16x8 lds_frag(const char* tile, int row, int chunk) {
  return *(const bf16x8*)(tile + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
}

// The value of lane l and of lane l ^ 32 (v_permlane32_swap: the upper half of one copy trades places with the lower
// half of the other, no trip through the LDS crossbar), combined with max or +.
__device__ __forceinline__ float half_wave_max(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_wave_sum(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// HD128 (ME_QKV_ROPE only): head_dim 128 instead of 64.
template <int BM, int EPI, int NWN, bool HD128 = false>
__global__ void __launch_bounds__(128 * NWN) gemm_mfma_kernel(GemmArgs a) {
  constexpr int BN = 256;
  // Rotary pairs are columns (i, i + hd/2) of a head. With head_dim 64 a wavefront's 64 columns are one head and
  // its two accumulator columns the two halves. With head_dim 128 a head spans two wavefronts, so the W tile is
  // loaded with rows 32..63 and 64..95 of every 128 exchanged: wavefront (head, wq) then holds columns
  // wq*32 .. +31 of the first half in accumulator column 0 and the same columns of the second half in column 1.
  constexpr bool SWAP = EPI == ME_QKV_ROPE && HD128;
  constexpr int NW = 2 * NWN;                         // wavefronts: 2 along M x NWN along N
  constexpr int WM = BM / 2, TM = WM / 32, WN = BN / NWN, TN = WN / 32;
  // All epilogues multiply W-fragment x A-fragment, i.e. the transposed 32x32 product: a lane then holds runs of
  // four consecutive COLUMNS of one row of C. The storing epilogues write them as one 16-byte (8-byte bf16) piece
  // (four times fewer store instructions than with single elements of four rows), and the vocabulary head reduces
  // its rows inside the lane instead of across lanes.
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // id -> (m_tile, n_tile): ids congruent mod 8 share an XCD. An XCD owns the N-tiles n = 8j + xcd; the 32
  // workgroups that run on it at one time form a block of 8 M-tiles x 4 of its N-tiles, so that every A panel
  // is fetched into that XCD's L2 once per 4 users and every W tile once per 8 users.
  const int id = blockIdx.x;
  const int xcd = id & 7, seq = id >> 3;
  const int blk = seq >> 5, within = seq & 31;
  const int m_tile = (blk % a.m_blocks) * 8 + (within & 7);
  const int n_tile = ((blk / a.m_blocks) * 4 + (within >> 3)) * 8 + xcd;
  if (n_tile >= a.n_tiles || m_tile >= a.m_tiles) return;
  const int m0 = m_tile * BM, n0 = n_tile * BN;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / NWN, wn = wave % NWN;
  const int lrow = lane & 31, lhalf = lane >> 5;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // K-tiles [kt0, kt0 + KT) of this workgroup's K slice
  const int kt0 = (int)((long)blockIdx.y * (a.K / 64) / a.ksplit);
  const int KT = (int)((long)(blockIdx.y + 1) * (a.K / 64) / a.ksplit) - kt0;
  // LDS ring of five slots; a slot holds one operand tile (A: BM x 64, W: 256 x 64). K-tile t uses slot 2t for
  // W and slot 2t+1 for A (mod 5), so besides the two slots being multiplied three are in flight: the weights,
  // which stream from HBM, are requested about two K-tiles ahead, the activations about one.
  constexpr int SLOT = 256 * 128;
  // phase = K-tile index mod 5; the k-loop is unrolled five times so that every slot address is a constant
  auto wslot = [&](int ph) { return smem + ((2 * ph) % 5) * SLOT; };
  auto aslot = [&](int ph) { return smem + ((2 * ph + 1) % 5) * SLOT; };
  // Measurement builds only (-DGEMM_ABLATE=bits, never defined in the library that ships): what the loop costs without
  // one of its parts. 1: no fragment reads after the first, 2: no workgroup barrier, 4: no operand loads after the
  // prologue. Results are wrong by construction; every access stays where it was and no wait is added.
#ifndef GEMM_ABLATE
#define GEMM_ABLATE 0
#endif
  bool in_prologue = true;
  auto read_frags = [&](int ph, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
    if ((GEMM_ABLATE & 1) && !in_prologue) return;
    const char* As = aslot(ph);
    const char* Bs = wslot(ph);
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = lds_frag(As, wm * WM + i * 32 + lrow, ks * 2 + lhalf);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = lds_frag(Bs, wn * WN + j * 32 + lrow, ks * 2 + lhalf);
  };
  auto mma = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
  };
  constexpr int LA = BM / (8 * NW), LB = BN / (8 * NW);   // direct-to-LDS loads per thread per operand tile
  auto issue_w = [&](int t) {                           // prologue only: t < 5 is its own phase
    const int src = t < KT ? t : KT - 1;
#pragma unroll
    for (int i = 0; i < LB; ++i) load_span_async<NW, SWAP>(a.W, n0, a.N, a.K, (kt0 + src) * 64, wslot(t), i, wave);
  };
  auto issue_a = [&](int t) {
    const int src = t < KT ? t : KT - 1;
#pragma unroll
    for (int i = 0; i < LA; ++i) load_span_async<NW>(a.A, m0, a.M, a.K, (kt0 + src) * 64, aslot(t), i, wave);
  };
  constexpr int NLD = LA + LB;
  auto share_size = [](int sh) { int c = 0; for (int j = 0; j < NLD; ++j) c += (j * 4 / NLD == sh); return c; };
  constexpr int S0 = share_size(0), S1 = share_size(1), S2 = share_size(2), S3 = share_size(3);
  static_assert(LB == 4 && (S0 == 2) && S1 <= 2 && S2 <= 2 && S3 <= 2, "the waits below are written for these counts");
  // share SH of the loads of A-tile ta (phase pa) and W-tile tw (phase pw)
  auto issue_share = [&](int ta, int pa, int tw, int pw, auto share) {
    constexpr int SH = decltype(share)::value;
    if ((GEMM_ABLATE & 4) && !in_prologue) return;
    const int sa = ta < KT ? ta : KT - 1, sw = tw < KT ? tw : KT - 1;   // past the end: redundant loads into free slots
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      if (j * 4 / NLD != SH) continue;
      if (j < LA) load_span_async<NW>(a.A, m0, a.M, a.K, (kt0 + sa) * 64, aslot(pa), j, wave);
      else load_span_async<NW, SWAP>(a.W, n0, a.N, a.K, (kt0 + sw) * 64, wslot(pw), j - LA, wave);
    }
  };
#define SGB __builtin_amdgcn_sched_group_barrier
#define PIPE_GROUP_ORDER(NLOADS)                                                                                   \
  SGB(0x008, 2, 0);                                                                                                \
  SGB(0x100, TM + TN, 0);                                                                                          \
  if (NLOADS == 1) { SGB(0x008, 3, 0); SGB(0x010, 1, 0); SGB(0x008, TM * TN - 5, 0); }                             \
  else if (NLOADS == 2) { SGB(0x008, 1, 0); SGB(0x010, 1, 0); SGB(0x008, 3, 0); SGB(0x010, 1, 0); SGB(0x008, TM * TN - 6, 0); } \
  else SGB(0x008, TM * TN - 2, 0);                                                                                 \
  __builtin_amdgcn_sched_barrier(0)

  issue_w(0); issue_a(0); issue_w(1);
  issue_share(1, 1, 2, 2, std::integral_constant<int, 0>{});
  asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
  bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
  read_frags(0, 0, a0, b0);
  if (GEMM_ABLATE) read_frags(0, 1, a1, b1);
  in_prologue = false;
  auto step = [&](auto phase, int kt) {
    constexpr int P = decltype(phase)::value;
    constexpr int P1 = (P + 1) % 5, P2 = (P + 2) % 5, P3 = (P + 3) % 5;
    read_frags(P, 1, a1, b1);
    issue_share(kt + 1, P1, kt + 2, P2, std::integral_constant<int, 1>{});
    mma(a0, b0);
    PIPE_GROUP_ORDER(S1);
    read_frags(P, 2, a0, b0);
    issue_share(kt + 1, P1, kt + 2, P2, std::integral_constant<int, 2>{});
    mma(a1, b1);
    PIPE_GROUP_ORDER(S2);
    read_frags(P, 3, a1, b1);
    issue_share(kt + 1, P1, kt + 2, P2, std::integral_constant<int, 3>{});
    mma(a0, b0);
    PIPE_GROUP_ORDER(S3);
    if (GEMM_ABLATE & 2) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
    else if (GEMM_ABLATE & 4) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    issue_share(kt + 2, P2, kt + 3, P3, std::integral_constant<int, 0>{});
    read_frags(P1, 0, a0, b0);                         // after the last K-tile: a read of a free slot, never used
    mma(a1, b1);
    PIPE_GROUP_ORDER(S0);
  };
  for (int kt = 0;;) {
    step(std::integral_constant<int, 0>{}, kt); if (++kt >= KT) break;
    step(std::integral_constant<int, 1>{}, kt); if (++kt >= KT) break;
    step(std::integral_constant<int, 2>{}, kt); if (++kt >= KT) break;
    step(std::integral_constant<int, 3>{}, kt); if (++kt >= KT) break;
    step(std::integral_constant<int, 4>{}, kt); if (++kt >= KT) break;
  }
#undef PIPE_GROUP_ORDER
#undef SGB
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // accumulator element r of a lane: row lrow, column 8*(r/4) + 4*lhalf + r%4 of the 32x32 tile
  if (EPI == ME_STORE || EPI == ME_RESIDUAL) {
    float* __restrict__ Cs = a.C + (size_t)blockIdx.y * a.M * a.N;
    const bool vec = (a.N & 3) == 0 && ((uintptr_t)a.C & 15) == 0;   // 16-byte pieces stay aligned and inside a row
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = m0 + wm * WM + i * 32 + lrow;
      if (row >= a.M) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int col = n0 + wn * WN + j * 32 + 8 * g + 4 * lhalf;
          float* dst = Cs + (size_t)row * a.N + col;
          if (vec && col + 3 < a.N) {
            float4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
            if (EPI == ME_RESIDUAL) {
              float4 o = *(const float4*)dst;
              v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
            }
            *(float4*)dst = v;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (col + e < a.N) {
                if (EPI == ME_RESIDUAL) dst[e] += acc[i][j][4 * g + e];
                else dst[e] = acc[i][j][4 * g + e];
              }
          }
        }
    }
  } else if (EPI == ME_SWIGLU) {
    const int F = a.N >> 1;                            // a multiple of 32: whole 4-unit pieces
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    // one decision for the workgroup: a tile inside the matrix stores without per-piece bounds checks
    const bool inside = m0 + BM <= a.M && n0 + BN <= a.N;
    auto emit = [&](auto checked) {
      constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
      for (int jp = 0; jp < TN / 2; ++jp) {            // accumulator pair (2jp, 2jp+1) = gate, up of 32 units
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int row = m0 + wm * WM + i * 32 + lrow;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int unit = ((n0 + wn * WN + jp * 64) >> 1) + 8 * g + 4 * lhalf;
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float gt = acc[i][2 * jp][4 * g + e], u = acc[i][2 * jp + 1][4 * g + e];
              // v_rcp_f32 (1 ulp) instead of an IEEE division: the quotient is rounded to bf16 right away, and the
              // division's scale/fix-up sequence alone was ten instructions per value
              o[e] = (__bf16)(gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * u);
            }
            if (!CHECK || (row < a.M && unit < F)) *(bf16x4*)(a.act + (size_t)row * F + unit) = o;
          }
        }
      }
    };
    if (inside) emit(std::false_type{});
    else emit(std::true_type{});
  } else if (EPI == ME_QKV_ROPE) {
    static_assert(EPI != ME_QKV_ROPE || (TN == 2 && NWN == 4), "one rotary half per accumulator column");
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    constexpr int HDIM = HD128 ? 128 : 64, HALF = HDIM / 2;
    const int head = HD128 ? (n0 >> 7) + (wn >> 1) : (n0 >> 6) + wn;
    const int i_base = (HD128 ? (wn & 1) * 32 : 0) + 4 * lhalf;          // + 8 g + e: index of the pair inside the head
    if (head < a.Hq + 2 * a.Hkv) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * WM + i * 32 + lrow;
        if (row >= a.M) continue;
        const int cand = row / a.Lrows, t = a.t0 + (row - cand * a.Lrows);
        if (head < a.Hq + a.Hkv) {
          const float* cs = a.cs + (size_t)row * HDIM;
          bf16_t* dst = head < a.Hq ? a.q + ((size_t)row * a.Hq + head) * HDIM
                                    : a.kblk + (((size_t)cand * a.Lk + t) * a.Hkv + (head - a.Hq)) * HDIM;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int i0 = i_base + 8 * g;
            const float4 cn = *(const float4*)(cs + i0), sn = *(const float4*)(cs + HALF + i0);
            const float c4[4] = {cn.x, cn.y, cn.z, cn.w}, s4[4] = {sn.x, sn.y, sn.z, sn.w};
            bf16x4 y1, y2;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float x1 = acc[i][0][4 * g + e], x2 = acc[i][1][4 * g + e];
              y1[e] = (__bf16)(x1 * c4[e] - x2 * s4[e]);
              y2[e] = (__bf16)(x2 * c4[e] + x1 * s4[e]);
            }
            *(bf16x4*)(dst + i0) = y1;
            *(bf16x4*)(dst + HALF + i0) = y2;
          }
        } else {
          // values: not rotated, stored transposed; the 32 lanes of a half-wave write 32 consecutive positions
          bf16_t* dst = a.vT + (((size_t)cand * a.Hkv + (head - a.Hq - a.Hkv)) * HDIM) * a.Lp + t;
          const bool pad = t == a.Lk - 1 && a.Lp > a.Lk;
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int d = i_base + 8 * g + e;
              dst[(size_t)d * a.Lp] = (__bf16)acc[i][0][4 * g + e];
              dst[(size_t)(HALF + d) * a.Lp] = (__bf16)acc[i][1][4 * g + e];
              if (pad)
                for (int tt = 1; tt < a.Lp - t; ++tt) {
                  dst[(size_t)d * a.Lp + tt] = (__bf16)0.f;
                  dst[(size_t)(HALF + d) * a.Lp + tt] = (__bf16)0.f;
                }
            }
        }
      }
    }
  } else {  // ME_LMHEAD
    __syncthreads();                                   // every wavefront is done with the operand tiles
    float* red_max = (float*)smem;                     // [BM][NWN]
    float* red_sum = red_max + BM * NWN;
    // A lane owns row lrow of each of its TM row tiles and, of the wavefront's WN columns, the 16 * TN with
    // (column / 4) % 2 == lhalf: maximum and sum of exponentials run over the lane's own registers, one exchange
    // joins the two half-waves, and the row's target column is looked for among the same registers.
    const bool ragged = n0 + BN > a.N;                 // only the last N-tile has columns beyond the matrix
    const int cbase = n0 + wn * WN + 4 * lhalf;        // column of element (j, r): cbase + 32 j + 8 (r / 4) + r % 4
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int lr = wm * WM + i * 32 + lrow, row = m0 + lr;
      const int target = row < a.M ? a.tok[row] : -1;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (ragged && cbase + 32 * j + 8 * (r >> 2) + (r & 3) >= a.N) acc[i][j][r] = -INFINITY;
          mx = fmaxf(mx, acc[i][j][r]);
        }
      mx = half_wave_max(mx);
      // the target's offset among this lane's columns; element (j, r) sits at 32 j + 8 (r / 4) + r % 4
      const int d = target - cbase;
      float sm = 0.f, zt = 0.f;
      bool hit = false;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float v = acc[i][j][r];
          sm += mx == -INFINITY ? 0.f : __expf(v - mx);
          const bool here = d == 32 * j + 8 * (r >> 2) + (r & 3);
          zt = here ? v : zt;
          hit |= here;
        }
      sm = half_wave_sum(sm);
      if (hit) a.zt[row] = zt;
      if (lhalf == 0) {
        red_max[lr * NWN + wn] = mx;
        red_sum[lr * NWN + wn] = sm;
      }
    }
    __syncthreads();
    for (int lr = threadIdx.x; lr < BM; lr += 64 * NW) {
      int row = m0 + lr;
      if (row < a.M) {
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < NWN; ++w) mx = fmaxf(mx, red_max[lr * NWN + w]);
        float sm = 0.f;
#pragma unroll
        for (int w = 0; w < NWN; ++w)
          if (red_max[lr * NWN + w] > -INFINITY) sm += red_sum[lr * NWN + w] * expf(red_max[lr * NWN + w] - mx);
        a.part_max[(size_t)row * a.n_tiles + n_tile] = mx;
        a.part_sum[(size_t)row * a.n_tiles + n_tile] = sm;
      }
    }
  }
}

template <int BM, int EPI, int NWN, bool HD128 = false>
static void launch_variant(const GemmArgs& a, hipStream_t s) {
  constexpr int smem = 5 * 256 * 128;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, EPI, NWN, HD128>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    configured = true;
  }
  int per_xcd = (a.n_tiles + 7) / 8;                 // N-tiles owned by one XCD
  int blocks = a.m_blocks * ((per_xcd + 3) / 4);     // 8 x 4 blocks per XCD
  gemm_mfma_kernel<BM, EPI, NWN, HD128><<<dim3(blocks * 32 * 8, a.ksplit), 128 * NWN, smem, s>>>(a);
}

int mfma_lmhead_tiles(int V) { return (V + 255) / 256; }

// Tile height and K-split for an M x N x K product whose consumer can sum partial products. Times in
// microseconds from measurements on the 256-CU part: one 64-deep k-step of a resident workgroup costs c(BM),
// workgroups run in rounds of 256, a launch has a fixed cost, and every extra partial costs one more
// M x N float write here plus one read in the consumer.
void mfma_gemm_plan(int M, int N, int K, int max_split, int* bm_out, int* split_out) {
  const int KT = K / 64, n_tiles = (N + 255) / 256;
  double best = 1e30;
  *bm_out = 256; *split_out = 1;
  for (int bm = M <= 128 ? 128 : 256; bm >= 128; bm >>= 1) {
    long tiles = (long)((M + bm - 1) / bm) * n_tiles;
    double c = bm == 256 ? 1.55 : 1.08;
    for (int sp = 1; sp <= max_split && sp <= 8 && sp * 4 <= KT + 3; ++sp) {
      long rounds = (tiles * sp + 255) / 256;
      double t = (double)rounds * ((KT + sp - 1) / sp) * c + 8.0 + (2 * sp - 2) * (double)M * N * 4.0 / 4e6;
      if (t < best - 1e-9) { best = t; *bm_out = bm; *split_out = sp; }
    }
  }
}

// QKV projection with the rotary embedding, the bf16 conversion and the per-candidate transposition of the values
// in the epilogue: no float [M, (Hq+2Hkv)*hd] round trip through memory and no separate kernel. Row m is in-block
// position g.t0 + m % g.L of candidate m / g.L. Returns false when the shape is not taken (head_dim other than
// 64/128, K % 64 != 0, misaligned buffers); the caller then runs the projection and the rotary kernel separately.
bool launch_gemm_mfma_qkv_rope(const bf16_t* A, const bf16_t* W, const float* cs, bf16_t* q, bf16_t* kblk, bf16_t* vT,
                               const BatchGeom& g, const ModelDims& md, int Lp, hipStream_t s) {
  const int M = g.M, N = (md.Hq + 2 * md.Hkv) * md.hd, K = md.d;
  if (K % 64 != 0 || M <= 0 || (md.hd != 64 && md.hd != 128)) return false;
  if (((uintptr_t)cs & 15) || ((uintptr_t)q & 7) || ((uintptr_t)kblk & 7)) return false;
  GemmArgs a = {};
  a.A = A; a.W = W; a.M = M; a.N = N; a.K = K; a.ksplit = 1;
  a.cs = cs; a.q = q; a.kblk = kblk; a.vT = vT;
  a.Hq = md.Hq; a.Hkv = md.Hkv; a.hd = md.hd; a.Lrows = g.L; a.t0 = g.t0; a.Lk = g.Lk; a.Lp = Lp;
  a.n_tiles = (N + 255) / 256;
  bool small = ((M + 255) / 256) * a.n_tiles <= 128 || M <= 128;
  a.m_tiles = small ? (M + 127) / 128 : (M + 255) / 256;
  a.m_blocks = (a.m_tiles + 7) / 8;
  if (md.hd == 128) { if (small) launch_variant<128, ME_QKV_ROPE, 4, true>(a, s); else launch_variant<256, ME_QKV_ROPE, 4, true>(a, s); }
  else { if (small) launch_variant<128, ME_QKV_ROPE, 4, false>(a, s); else launch_variant<256, ME_QKV_ROPE, 4, false>(a, s); }
  return true;
}

// Returns false when the shape is not one this kernel takes (the caller then uses the SIMT kernel).
// ksplit > 1 (ME_STORE only): C is [ksplit][M][N] and receives the partial products of the K slices.
// bm: tile height 128 or 256, 0 = chosen here.
bool launch_gemm_mfma(int epi, const bf16_t* A, const bf16_t* W, int M, int N, int K, float* C, bf16_t* act,
                      const int32_t* tok, float* part_max, float* part_sum, float* zt, int ksplit, int bm,
                      hipStream_t s) {
  if (K % 64 != 0 || M <= 0 || N <= 0) return false;
  if (epi == ME_SWIGLU && (N % 64 != 0 || ((uintptr_t)act & 7))) return false;
  if (ksplit < 1 || (ksplit > 1 && (epi != ME_STORE || ksplit > K / 64))) return false;
  if (bm != 0 && bm != 128 && bm != 256) return false;
  GemmArgs a = {};
  a.A = A; a.W = W; a.M = M; a.N = N; a.K = K; a.C = C; a.act = act; a.tok = tok;
  a.part_max = part_max; a.part_sum = part_sum; a.zt = zt; a.ksplit = ksplit;
  a.n_tiles = (N + 255) / 256;
  // 128-row tiles when twice as many workgroups still fit the 256 CUs in one round
  bool small = bm ? bm == 128 : ((M + 255) / 256) * a.n_tiles <= 128 || M <= 128;
  a.m_tiles = small ? (M + 127) / 128 : (M + 255) / 256;
  a.m_blocks = (a.m_tiles + 7) / 8;
#define DISPATCH(E)                                                       \
  if (small) launch_variant<128, E, 4>(a, s);                             \
  else launch_variant<256, E, 4>(a, s);
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
