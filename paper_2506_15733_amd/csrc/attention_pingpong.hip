// Shared-prefix paged attention for whole blocks, two-phase ("ping-pong") schedule (bf16, head_dim 64 or 128,
// 16-token pages).
//
// Rows. For one beam b and kv head, the queries of ALL n candidates are stacked: row r = i*(L*g) + t*g + j is
// query head kvh*g + j of token t of candidate i (g = Hq/Hkv). All of these rows read the same prefix keys, so a
// workgroup takes 256 consecutive rows whatever candidates they belong to: a key/value tile staged into LDS once
// serves 256 rows (one workgroup per CU, eight wavefronts of 32 rows), and there is no padding when L*g is not a
// multiple of the tile height. The candidates' own block keys come after the prefix: the workgroup walks the
// block tiles of every candidate that owns one of its rows, and a lane masks the keys of other candidates and the
// keys after its own token.
//
// Schedule. The per-tile work of a wavefront is a matrix part (O^T += V^T P^T of the previous tile, then
// S^T = K Q^T of this tile: 8*HD/32 MFMAs) and a vector part (the softmax of S: maxima, exponentials, sums,
// bf16 packing), about equally long, and inside one wavefront they are serial. The eight wavefronts form two
// groups that share the four SIMDs pairwise and run half a tile apart: while group 0 is in its matrix part, group
// 1 is in its vector part, exchanged at a workgroup barrier, so that on every SIMD the matrix pipe and the vector
// ALU are busy at the same time instead of whenever two independent workgroups happen to drift apart.
//
// Tiles are staged global -> LDS directly (16 bytes per lane) into a ring of four slots, two tiles ahead of their
// use, by the group that is in its vector part (group 1 loads keys, group 0 values); a slot is rewritten only
// after both groups have multiplied its values.
//
// Arithmetic per tile is the flash-attention recurrence of the one-phase kernel (attention_mfma.hip): transposed
// products so that a lane owns a query column, integer reference exponents that follow the running maximum lazily.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Measurement builds only (-DATTN_ABLATE=bits, never defined in the library that ships): the kernel without one of
// its parts. 1: no softmax arithmetic (scores are converted to bf16 as they are), 2: no staging loads after the first
// two tiles, 4: no fragment reads from LDS (one register value serves as every fragment). Results are wrong by
// construction; every access that remains stays where it was and no wait is added.
#ifndef ATTN_ABLATE
#define ATTN_ABLATE 0
#endif

namespace {

constexpr int kMaxBlockTiles = 1024;   // block tiles one workgroup can list (entries of its LDS table)
constexpr int kMaxPages = 4096;        // pages of one beam's prefix (entries of the workgroup's LDS copy of its page table)

struct PPArgs {
  const bf16_t* q;      // [M][Hq][hd]
  const bf16_t* kb;     // [M][Hkv][hd] block keys
  const bf16_t* vbT;    // [B*n][Hkv][hd][Lp] block values, transposed, zero padded
  const bf16_t* poolK;  // [pages][Hkv][16][hd]
  const bf16_t* poolV;  // [pages][Hkv][hd][16]
  bf16_t* out;          // [M][Hq*hd]
  BatchGeom g;
  int Hq, Hkv, Lp, wg_tiles, total_wg, wg_per_xcd;
  int balanced;         // (beam, kv head) units dealt to the XCDs by decreasing prefix length (see the kernel)
  float scale_log2e;
  int n_splits;         // > 1: the prefix tiles are cut into runs, the last run also takes the block tiles; every
  float* part_o;        //      workgroup leaves (O un-normalised, m, l) per row for the merge kernel:
  float* part_m;        //      [(b*Hkv + kvh)][wg_tile][split][256] rows, part_o [..][HD]
  float* part_l;
};

__device__ __forceinline__ float half_wave_max(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_wave_sum(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int HD>
__device__ __forceinline__ int k_swizzle(int row, int chunk) {
  return HD == 128 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
}

template <int HD>
__global__ void __launch_bounds__(512, 2) attention_pingpong_kernel(PPArgs a) {
  constexpr int KROW = HD * 2;              // bytes per key row
  constexpr int KCH = HD / 8;               // 16-byte chunks per key row
  constexpr int K_BYTES = 64 * KROW;        // 64 keys
  constexpr int V_BYTES = 4 * HD * 32;      // 4 groups of [HD][16]
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int NSTAGE = 4;
  constexpr int NI = HD / 32;               // 1 KiB load instructions per 16-key group and operand; also d-tiles
  constexpr int SHARE = NI;                 // load instructions per wavefront and tile (one operand of one 16-key group)
  constexpr int KS = HD / 16;               // MFMA K-steps of the S^T product
  constexpr int BQ = 256;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const BatchGeom& G = a.g;
  const int g = a.Hq / a.Hkv;
  // Workgroup -> (beam, kv head, row tile, run). Workgroups whose ids are congruent mod 8 share an XCD, and all
  // workgroups of a (beam, kv head) go to one XCD, whose L2 then fetches that head's pages once.
  int b, kvh, rem;
  if (a.balanced) {
    // Ragged batches: a workgroup's duration follows its beam's prefix length, so the (beam, kv head) units are dealt
    // to the XCDs in order of decreasing length, back and forth (ranks 0..7, then 15..8, ...): every XCD gets the same
    // sum to within a unit and starts with its longest ones. The rank -> beam look-up is recomputed by every
    // wavefront (at most 64 beams).
    const int per_unit = a.wg_tiles * a.n_splits;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int pos = slot / per_unit;
    rem = slot - pos * per_unit;
    const int unit_rank = (pos & 1) ? pos * 8 + 7 - xcd : pos * 8 + xcd;
    if (unit_rank >= G.B * a.Hkv) return;
    const int rank = unit_rank / a.Hkv;
    kvh = unit_rank - rank * a.Hkv;
    const int ln = threadIdx.x & 63;
    const int mine = ln < G.B ? G.lens[G.b0 + ln] : -1;
    int r = 0;
    for (int i = 0; i < G.B; ++i) {
      const int other = __shfl(mine, i, 64);
      r += (other > mine || (other == mine && i < ln)) ? 1 : 0;
    }
    const unsigned long long hit = __ballot(ln < G.B && r == rank);      // ranks are distinct: exactly one lane
    b = __builtin_amdgcn_readfirstlane(__ffsll((long long)hit) - 1);
  } else {
    const int logical = (blockIdx.x & 7) * a.wg_per_xcd + (blockIdx.x >> 3);
    if (logical >= a.total_wg) return;
    b = logical / (a.Hkv * a.wg_tiles * a.n_splits);
    rem = logical - b * (a.Hkv * a.wg_tiles * a.n_splits);
    kvh = rem / (a.wg_tiles * a.n_splits);
    rem -= kvh * (a.wg_tiles * a.n_splits);
  }
  const int split = rem % a.n_splits;
  const int wg_tile = rem / a.n_splits;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int grp = wave >> 2;                 // wavefronts w and w + 4 share a SIMD and belong to different groups
  const int lq = lane & 31, lh = lane >> 5;
  const int P = G.len_override >= 0 ? G.len_override : G.lens[G.b0 + b];
  const int L = G.L, Lg = L * g;
  const int R = G.n * Lg;                    // stacked rows of this (beam, kv head)
  const int r_wg0 = wg_tile * BQ;
  const int r_wg1 = (r_wg0 + BQ - 1 < R - 1) ? r_wg0 + BQ - 1 : R - 1;      // last valid row of the workgroup
  const int32_t* ptab = G.page_table + (size_t)(G.b0 + b) * G.max_pages;

  // this lane's query row
  const int r_lane = r_wg0 + wave * 32 + lq;
  const int rc = r_lane < R ? r_lane : R - 1;
  const int cand_lane = rc / Lg;
  const int rr = rc - cand_lane * Lg;
  const int t_lane = rr / g, j_lane = rr - t_lane * g;
  const size_t m_lane = ((size_t)b * G.n + cand_lane) * L + t_lane;
  // rows of this wavefront (scalars): candidates and the last token they reach
  const int rw0 = __builtin_amdgcn_readfirstlane(r_wg0 + wave * 32 < R ? r_wg0 + wave * 32 : R - 1);
  const int rw1 = __builtin_amdgcn_readfirstlane(r_wg0 + wave * 32 + 31 < R ? r_wg0 + wave * 32 + 31 : R - 1);

  bf16x8 qf[KS];
  {
    const bf16_t* src = a.q + (m_lane * a.Hq + (size_t)kvh * g + j_lane) * HD;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(src + ks * 16 + lh * 8);
    // the staging loads below are counted: nothing older may still be in flight when the counting starts
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  floatx16 o[NI];
#pragma unroll
  for (int dt = 0; dt < NI; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- tile list of this workgroup: prefix tiles [pt_lo, pt_lo + npt), then the block tiles of its candidates
  const int n_ptiles = (P + 63) >> 6;
  const int n_pages = (P + 15) >> 4;
  const int pt_lo = (int)((long)split * n_ptiles / a.n_splits);
  const int npt = (int)((long)(split + 1) * n_ptiles / a.n_splits) - pt_lo;
  const int c_lo = r_wg0 / Lg, c_hi = r_wg1 / Lg;
  // block tiles of candidate c that some row of the workgroup can see: 0 .. (last token of c among the rows) / 64
  auto block_tiles_of = [&](int c) {
    int last = (c + 1) * Lg - 1;
    last = last < r_wg1 ? last : r_wg1;
    return (((last - c * Lg) / g) >> 6) + 1;
  };
  int T = npt;
  if (split == a.n_splits - 1)
    for (int c = c_lo; c <= c_hi; ++c) T += block_tiles_of(c);

  // The block tiles (candidate, tile number) are listed once in LDS behind the staging ring; the tile loop looks an
  // entry up instead of walking the candidates again for every tile (an instruction a wavefront issues costs four
  // clocks whatever it is, and the matrix part of a tile has only a few hundred to spare).
  // The beam's page numbers are copied to LDS as well: a scalar load inside the tile loop would share the LDS
  // counter, complete out of order and force every fragment wait that follows it to wait for everything.
  int* tile_table = (int*)(smem + NSTAGE * STAGE);
  int* page_lds = tile_table + kMaxBlockTiles;
  for (int i = threadIdx.x; i < n_pages; i += 512) page_lds[i] = ptab[i];
  if (threadIdx.x == 0 && T > npt) {
    int k = 0;
    for (int c = c_lo; c <= c_hi; ++c) {
      const int nb = block_tiles_of(c);
      for (int i = 0; i < nb; ++i) tile_table[k++] = c | (i << 16);
    }
  }
  __syncthreads();
  struct Tile { bool is_block; int c, idx; };          // idx: prefix tile number, or block tile number of candidate c
  auto tile_at = [&](int tau) {
    Tile t;
    if (tau < npt) { t.is_block = false; t.c = 0; t.idx = pt_lo + tau; return t; }
    const int e = __builtin_amdgcn_readfirstlane(tile_table[tau - npt]);
    t.is_block = true; t.c = e & 0xffff; t.idx = e >> 16;
    return t;
  };
  // does this wavefront have a row that sees a key of the tile?
  auto wave_active = [&](const Tile& t) {
    if (!t.is_block) return true;
    const int lo = t.c * Lg, hi = (t.c + 1) * Lg - 1;
    if (rw1 < lo || rw0 > hi) return false;
    const int last = (rw1 < hi ? rw1 : hi) - lo;         // last row of candidate c in this wavefront
    return t.idx * 64 <= last / g;
  };

  // ---- staging: a wavefront loads one operand of 16-key group (w & 3) of a tile: group 1 the keys, group 0 the
  // values. Each group issues its loads at the start of its own softmax phase, so that the wavefronts that are
  // multiplying never queue behind the vector-memory issue of eight wavefronts at once.
  const int pg = wave & 3;
  const bool loads_keys = grp == 1;
  auto page_of = [&](int tau) -> int {
    if (tau >= npt) return 0;
    int p16 = (pt_lo + tau) * 4 + pg;
    p16 = p16 < n_pages ? p16 : n_pages - 1;
    return __builtin_amdgcn_readfirstlane(page_lds[p16]);
  };
  // lane offsets of the prefix-page loads (elements): the same for every tile, kept in registers
  unsigned p_off[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int qi = i * 64 + lane;
    const int row = qi / KCH, slot = qi % KCH;
    const int d = qi >> 1, half = (qi & 1) ^ ((d >> 3) & 1);     // LDS chunk position qi&1 holds key half `half`
    p_off[i] = loads_keys ? (unsigned)(row * HD + k_swizzle<HD>(pg * 16 + row, slot) * 8) : (unsigned)(d * 16 + half * 8);
  }
  auto stage_part = [&](int tau, int page_id) {
    if ((ATTN_ABLATE & 2) && tau >= 2) return;
    char* buf = smem + (tau % NSTAGE) * STAGE;
    char* dst = loads_keys ? buf + pg * 16 * KROW : buf + K_BYTES + pg * HD * 32;
    const Tile t = tile_at(tau);
    if (!t.is_block) {
      size_t page = (size_t)__builtin_amdgcn_readfirstlane(page_id);
      const bf16_t* src = (loads_keys ? a.poolK : a.poolV) + (page * a.Hkv + kvh) * 16 * HD;
#pragma unroll
      for (int i = 0; i < NI; ++i)
        __builtin_amdgcn_global_load_lds(GLB_PTR(src + p_off[i]), LDS_PTR(dst + i * 1024), 16, 0, 0);
    } else {
      // block tiles are few: their addresses are recomputed per call from a lane id the compiler cannot see
      // through (hoisted out of the tile loop they would occupy registers for the whole kernel)
      int lane = threadIdx.x & 63;
      asm volatile("" : "+v"(lane));
      const size_t cidx = (size_t)b * G.n + t.c;
      const int key0 = t.idx * 64 + pg * 16;
      if (loads_keys) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          int qi = i * 64 + lane;
          int row = qi / KCH, slot = qi % KCH;
          int chunk = k_swizzle<HD>(pg * 16 + row, slot);
          int key = key0 + row;
          key = key < L ? key : L - 1;
          const bf16_t* src = a.kb + ((cidx * L + key) * a.Hkv + kvh) * HD + chunk * 8;
          __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(dst + i * 1024), 16, 0, 0);
        }
      } else {
        const bf16_t* vsrc = a.vbT + (cidx * a.Hkv + kvh) * HD * a.Lp;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          int qi = i * 64 + lane;
          int d = qi >> 1, half = (qi & 1) ^ ((d >> 3) & 1);
          int key = key0 + half * 8;
          key = key < a.Lp ? key : a.Lp - 8;
          __builtin_amdgcn_global_load_lds(GLB_PTR(vsrc + (size_t)d * a.Lp + key), LDS_PTR(dst + i * 1024), 16, 0, 0);
        }
      }
    }
  };

  // pi(i): A-row i of the S^T product carries key pi(i) of the 32-key half tile (see attention_mfma.hip)
  const int pi_row_c = (lq & 16) | ((lq & 4) << 1) | ((lq & 8) >> 1) | (lq & 3);
  const int lh_c = lh, lq_c = lq;

  floatx16 s[2];
  bf16x8 pf[4];

  // S^T = K Q^T of tile tau
  auto qk = [&](int tau) {
    const char* Ks = smem + (tau % NSTAGE) * STAGE;
    const int pi_row = pi_row_c, lh = lh_c;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[hf][r] = 0.f;
    constexpr int KPF = 4;
    auto read_kf = [&](int ks, int hf) {
      if (ATTN_ABLATE & 4) return qf[0];
      int row = hf * 32 + pi_row;
      return *(const bf16x8*)(Ks + row * KROW + (k_swizzle<HD>(row, ks * 2 + lh) << 4));
    };
    bf16x8 kf[KPF + 1][2];
#pragma unroll
    for (int ks = 0; ks < KPF; ++ks)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) kf[ks][hf] = read_kf(ks, hf);
    // fragments are read KPF steps ahead of the MFMAs that use them and no further (the scheduler would otherwise
    // hoist all reads to the top and hold every fragment in registers)
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * KPF, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + KPF < KS) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) kf[(ks + KPF) % (KPF + 1)][hf] = read_kf(ks + KPF, hf);
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        s[hf] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks % (KPF + 1)][hf], qf[ks], s[hf], 0, 0, 0);
      if (ks + KPF < KS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
  };

  // softmax of tile tau: s -> pf, (m_run, l_run), rescale of o when the reference exponent moves
  auto softmax = [&](const Tile& t) {
    if (ATTN_ABLATE & 1) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int r = 0; r < 16; ++r) pf[hf * 2 + (r >> 3)][r & 7] = (bf16_t)s[hf][r];
      l_run = 1.f;
      return;
    }
    const int key_base = t.idx * 64;
    // accumulator value r of half hf in this lane is key  key_base + hf*32 + 16*(r/8) + 8*lh + r%8
    const bool need_mask = t.is_block || (key_base + 64 > P);
    if (need_mask) {
      // keys < limit are visible: the prefix length, or (own candidate only) the lane's token + 1
      const int limit = t.is_block ? ((cand_lane == t.c && r_lane < R) ? t_lane + 1 : 0) : P;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int key = key_base + hf * 32 + 16 * (r >> 3) + 8 * lh + (r & 7);
          s[hf][r] = key < limit ? s[hf][r] : -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[hf][r]);
    mx = half_wave_max(mx);
    // integer reference exponent in the log2 domain, moved only when the maximum has outgrown it by 2^8
    constexpr float RESCALE_LOG2 = 8.f;
    const float m_tile = mx * a.scale_log2e;
    const bool move = m_tile > m_run + RESCALE_LOG2;       // also the first visible key: -inf + 8 = -inf
    if (__any(move)) {
      const float m_new = move ? ceilf(m_tile) : m_run;
      const float alpha = move ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;   // exp2(-inf) = 0: nothing yet
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < NI; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
      m_run = m_new;
    }
    const float m_use = m_run == -INFINITY ? 0.f : m_run;   // nothing visible yet: every p below is exp2(-inf) = 0
    float psum = 0.f;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(fmaf(s[hf][r], a.scale_log2e, -m_use));
        psum += p;
        pf[hf * 2 + (r >> 3)][r & 7] = (bf16_t)p;
      }
    l_run += psum;
  };

  // O^T += V^T P^T of tile tau: K-step = one 16-key group, this lane supplies keys 8*lh .. 8*lh+7 of it
  auto pv = [&](int tau) {
    const char* Vs = smem + (tau % NSTAGE) * STAGE + K_BYTES;
    const int lq = lq_c, lh = lh_c;
    constexpr int VPF = 8, NST = 4 * NI;
    auto read_vf = [&](int st) {
      if (ATTN_ABLATE & 4) return qf[1];
      const int p4 = st / NI, dt = st % NI;
      return *(const bf16x8*)(Vs + p4 * HD * 32 + (dt * 32 + lq) * 32 + ((lh ^ ((lq >> 3) & 1)) << 4));
    };
    bf16x8 vf[VPF + 1];
#pragma unroll
    for (int st = 0; st < VPF; ++st) vf[st] = read_vf(st);
    __builtin_amdgcn_sched_group_barrier(0x100, VPF, 0);
#pragma unroll
    for (int st = 0; st < NST; ++st) {
      const int p4 = st / NI, dt = st % NI;
      if (st + VPF < NST) vf[(st + VPF) % (VPF + 1)] = read_vf(st + VPF);
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[st % (VPF + 1)], pf[p4], o[dt], 0, 0, 0);
      if (st + VPF < NST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
  };

  // ---- prologue: this wavefront's operand of tiles 0 and 1 in flight, that of tile 0 landed
  int page_next = 0;
  if (T > 0) stage_part(0, page_of(0));
  if (T > 1) stage_part(1, page_of(1));
  if (T > 2) page_next = page_of(2);
  if (T > 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(SHARE) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // Phases phi = 0 .. 2T+1, a workgroup barrier after each. Group 0 runs the matrix part of tile tau (values of tile
  // tau-1, keys of tile tau) in phase 2*tau and its softmax in phase 2*tau+1; group 1 does the same one phase later.
  // Group 1 requests the keys of tile tau+2 at the start of phase 2*tau, group 0 its values at the start of phase
  // 2*tau+1 (each at the start of a softmax phase of its own). The two groups run separate loops whose bodies are
  // straight-line (matrix part, softmax) so that scores and weights are short-lived values.
  auto stage_ahead = [&](int tl) {
    if (tl < T) {
      stage_part(tl, page_next);
      if (tl + 1 < T) page_next = page_of(tl + 1);
    }
  };
  auto end_odd = [&](int phi) {
    // Before phase phi + 1 = 2 * tn group 0 reads the keys of tile tn. The only request of this wavefront that is
    // younger than its part of tile tn is that for tile tn + 1, which may stay in flight.
    const int tn = (phi + 1) >> 1;
    if (tn + 1 < T) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(SHARE) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  auto matrix_part = [&](int tau) {
    if (tau >= 1 && wave_active(tile_at(tau - 1))) pv(tau - 1);
    if (tau < T && wave_active(tile_at(tau))) qk(tau);
  };
  auto vector_part = [&](int tau) {
    const Tile t = tile_at(tau);
    // the vector part is the longer of the two while the SIMD's other wavefront is issuing MFMAs: it goes first
    __builtin_amdgcn_s_setprio(2);
    if (wave_active(t)) softmax(t);
    __builtin_amdgcn_s_setprio(0);
  };
  if (grp == 0) {
    for (int tau = 0; tau < T; ++tau) {
      matrix_part(tau);
      __syncthreads();
      stage_ahead(tau + 2);                     // values of tile tau + 2, phase 2 * tau + 1
      vector_part(tau);
      end_odd(2 * tau + 1);
    }
    matrix_part(T);
    __syncthreads();
    end_odd(2 * T + 1);
  } else {
    stage_ahead(2);                             // keys of tile 2, phase 0
    __syncthreads();
    for (int tau = 0; tau < T; ++tau) {
      matrix_part(tau);
      end_odd(2 * tau + 1);
      stage_ahead(tau + 3);                     // keys of tile tau + 3, phase 2 * tau + 2
      vector_part(tau);
      __syncthreads();
    }
    matrix_part(T);
    end_odd(2 * T + 1);
  }

  // ---- normalise and store: lane = query column, accumulator value r of d-tile dt is d = dt*32 + 8*(r/4) + 4*lh + r%4
  const float l = half_wave_sum(l_run);
  if (a.n_splits > 1) {
    const size_t prow = ((((size_t)b * a.Hkv + kvh) * a.wg_tiles + wg_tile) * a.n_splits + split) * BQ + wave * 32 + lq;
    if (lh == 0) { a.part_m[prow] = m_run; a.part_l[prow] = l; }
    float* dst = a.part_o + prow * HD;
#pragma unroll
    for (int dt = 0; dt < NI; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        float4 v = {o[dt][r4 * 4], o[dt][r4 * 4 + 1], o[dt][r4 * 4 + 2], o[dt][r4 * 4 + 3]};
        *(float4*)(dst + dt * 32 + 8 * r4 + 4 * lh) = v;
      }
  } else if (r_lane < R) {
    const float inv = 1.0f / l;
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    bf16_t* dst = a.out + (m_lane * a.Hq + (size_t)kvh * g + j_lane) * HD;
#pragma unroll
    for (int dt = 0; dt < NI; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(o[dt][r4 * 4 + e] * inv);
        *(bf16x4*)(dst + dt * 32 + 8 * r4 + 4 * lh) = v;
      }
  }
}

// Merge of the partial results of a split launch: one wavefront per (row, query head).
template <int HD>
__global__ void __launch_bounds__(64) attention_pingpong_merge_kernel(const float* __restrict__ part_o,
                                                                      const float* __restrict__ part_m,
                                                                      const float* __restrict__ part_l,
                                                                      bf16_t* __restrict__ out, int n, int L, int Hq,
                                                                      int Hkv, int wg_tiles, int n_splits) {
  const size_t m = blockIdx.x;
  const int h = blockIdx.y, lane = threadIdx.x;
  const int g = Hq / Hkv, kvh = h / g, j = h - kvh * g;
  const size_t cand_idx = m / L;                           // b*n + i
  const int t = (int)(m - cand_idx * L);
  const size_t b = cand_idx / n, i = cand_idx - b * n;
  const size_t r = i * (size_t)L * g + (size_t)t * g + j;
  const size_t prow0 = (((b * Hkv + kvh) * wg_tiles + (r >> 8)) * n_splits) * 256 + (r & 255);   // + split*256
  float mx = -INFINITY;
  for (int s = 0; s < n_splits; ++s) mx = fmaxf(mx, part_m[prow0 + (size_t)s * 256]);
  float l = 0.f, acc[HD / 64];
#pragma unroll
  for (int u = 0; u < HD / 64; ++u) acc[u] = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const size_t pr = prow0 + (size_t)s * 256;
    const float w = __builtin_amdgcn_exp2f(part_m[pr] - mx);   // 0 for a run that saw no visible key
    l = fmaf(w, part_l[pr], l);
#pragma unroll
    for (int u = 0; u < HD / 64; ++u) acc[u] = fmaf(w, part_o[pr * HD + lane + 64 * u], acc[u]);
  }
  const float inv = 1.0f / l;
#pragma unroll
  for (int u = 0; u < HD / 64; ++u) out[(m * Hq + h) * HD + lane + 64 * u] = (bf16_t)(acc[u] * inv);
}

template <int HD>
void launch_pp_variant(const PPArgs& a, hipStream_t s) {
  constexpr int smem = 4 * (64 * HD * 2 + 4 * HD * 32) + (kMaxBlockTiles + kMaxPages) * 4;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)attention_pingpong_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              smem);
    configured = true;
  }
  attention_pingpong_kernel<HD><<<dim3(a.wg_per_xcd * 8), 512, smem, s>>>(a);
}

}  // namespace

// Whole-block launches (g.t0 == 0, g.Lk == g.L). Returns false if the shape is not taken (head_dim 64/128, 16-token
// pages, 8-byte aligned output rows). part / part_floats: float scratch for launches that cut the prefix into runs.
bool launch_attention_pingpong(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* poolK,
                               const bf16_t* poolV, bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp,
                               int max_ctx, float* part, size_t part_floats, hipStream_t s) {
  if ((md.hd != 64 && md.hd != 128) || g.page_tokens != 16 || Lp % 16 != 0 || g.t0 != 0 || g.Lk != g.L) return false;
  if (((uintptr_t)out & 7) || md.Hq % md.Hkv || g.n > 0xffff) return false;   // the tile table packs (candidate, tile) in 16 + 16 bits
  PPArgs a;
  a.q = q; a.kb = kb; a.vbT = vbT; a.poolK = poolK; a.poolV = poolV; a.out = out; a.g = g;
  a.Hq = md.Hq; a.Hkv = md.Hkv; a.Lp = Lp;
  a.scale_log2e = 1.4426950408889634f / sqrtf((float)md.hd);
  const long Lg = (long)g.L * (md.Hq / md.Hkv), rows = (long)g.n * Lg;
  const long cands_per_wg = 255 / Lg + 2 < g.n ? 255 / Lg + 2 : g.n;
  if (cands_per_wg * ((g.L + 63) / 64) > kMaxBlockTiles || (max_ctx + 15) / 16 > kMaxPages) return false;
  a.wg_tiles = (int)((rows + 255) / 256);
  const int base = g.B * md.Hkv * a.wg_tiles;
  // Few workgroups and a long prefix: cut the prefix tiles into runs so that about one workgroup per CU exists,
  // at least eight tiles per run, at most eight runs; a second kernel merges the partial results. (Measured: the
  // one-phase kernel's split mode, with 128-row workgroups, is faster for such launches; the caller prefers it.)
  const int prefix_tiles = (max_ctx + 63) / 64;
  int splits = 1;
  if (part && base < 160 && prefix_tiles >= 16) {
    splits = 256 / base;
    splits = splits > 8 ? 8 : splits;
    splits = splits > prefix_tiles / 8 ? prefix_tiles / 8 : splits;
    const size_t per_split = (size_t)base * 256 * (md.hd + 2);
    if (splits > 1 && (size_t)splits * per_split > part_floats) splits = (int)(part_floats / per_split);
    if (splits < 1) splits = 1;
  }
  a.n_splits = splits;
  a.part_o = nullptr; a.part_m = nullptr; a.part_l = nullptr;
  if (splits > 1) {
    const size_t rows_all = (size_t)base * splits * 256;
    a.part_o = part; a.part_m = part + rows_all * md.hd; a.part_l = a.part_m + rows_all;
  }
  a.total_wg = base * splits;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  a.balanced = g.B >= 16 && g.B <= 64 && g.len_override < 0;
  if (a.balanced) a.wg_per_xcd = ((g.B * md.Hkv + 7) / 8) * a.wg_tiles * splits;
  if (md.hd == 128) launch_pp_variant<128>(a, s); else launch_pp_variant<64>(a, s);
  if (splits > 1) {
    dim3 grid(g.M, md.Hq);
    if (md.hd == 128)
      attention_pingpong_merge_kernel<128><<<grid, 64, 0, s>>>(a.part_o, a.part_m, a.part_l, out, g.n, g.L, md.Hq,
                                                              md.Hkv, a.wg_tiles, splits);
    else
      attention_pingpong_merge_kernel<64><<<grid, 64, 0, s>>>(a.part_o, a.part_m, a.part_l, out, g.n, g.L, md.Hq,
                                                             md.Hkv, a.wg_tiles, splits);
  }
  return true;
}
