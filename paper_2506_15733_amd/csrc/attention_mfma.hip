// Shared-prefix paged attention on MFMA (bf16, head_dim 64 or 128, 16-token pages).
//
// Work decomposition. For one beam b, candidate i and kv head, the g = Hq/Hkv query heads of the
// L block tokens are stacked into L*g rows (row r = t*g + j: token t, query head kvh*g + j) that
// all read the same keys. A workgroup (4 wavefronts) owns 32*QT*4 of those rows and walks over
// the keys in tiles of 64: first the beam's cached prefix (4 pages per tile), then the
// candidate's own block (causal). The n candidates of a beam run as neighbouring workgroups on the
// same XCD, so the prefix pages are fetched from HBM once and re-read from L2.
//
// Per tile (flash-attention recurrence, float state):
//   S^T[key, q] = K Q^T   (MFMA 32x32x16, A = keys from LDS, B = queries held in registers)
//   m' = max(m, max_key S), alpha = exp(m - m'), p = exp(S - m'), l = l*alpha + sum p
//   O^T[d, q] = O^T*alpha + V^T P^T   (A = V^T from LDS, B = p rounded to bf16)
// In the transposed orientation a lane owns one query column, so the max over keys is a reduction
// over the lane's own 32 accumulator values plus one exchange with the other half-wave, and the
// rescale by alpha is a per-lane scalar.
//
// The A-rows of the S^T product are fed with keys in the order pi(i) (the two middle groups of
// four swapped inside every 16) so that the eight accumulator values a lane holds for one MFMA
// K-step of the second product are eight CONSECUTIVE keys: with V stored transposed
// ([head_dim][16 tokens] per page) the matching A-operand is one 16-byte LDS read. In LDS the two 16-byte
// halves of a V^T row are swapped for rows with bit 3 set, so that 16 consecutive lanes (rows 32 bytes apart,
// same half) cover all 64 banks instead of every other 16-byte column.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

struct AttnArgs {
  const bf16_t* q;      // [M][Hq][hd]
  const bf16_t* kb;     // [M][Hkv][hd] block keys
  const bf16_t* vbT;    // [B*n][Hkv][hd][Lp] block values, transposed, zero padded
  const bf16_t* poolK;  // [pages][Hkv][16][hd]
  const bf16_t* poolV;  // [pages][Hkv][hd][16]
  bf16_t* out;          // [M][Hq*hd]
  BatchGeom g;
  int Hq, Hkv, Lp, q_tiles, total_wg, wg_per_xcd;
  float scale_log2e;
  // single-position launches (generation): the prefix keys are cut into n_splits runs of tiles and every
  // workgroup leaves an un-normalised partial result for a second kernel to merge
  int n_splits;
  float* part_o;        // [(b*Hkv + kvh) (, candidate)][q_tile][split][128][HD]
  float* part_m;        // [..][128] running maximum (log2 domain), -inf if the run was empty
  float* part_l;        // [..][128] sum of weights relative to that maximum
};

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

template <int HD>
__device__ __forceinline__ int k_swizzle(int row, int chunk) {
  return HD == 128 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
}

// MODE 0: whole blocks, as described above. MODE 1: one position per candidate; the stacked rows of a
// (beam, kv head) are its n candidates x g query heads (row r = i*g + j), the workgroup covers only the prefix
// tiles of its split and writes (O un-normalised, m, l) instead of the output; the candidate's own block keys
// are added by the merge kernel. MODE 2: whole blocks, but the tile list (prefix tiles, then block tiles) is cut
// into n_splits runs handled by different workgroups, for launches that would otherwise leave most CUs idle; a
// merge kernel combines the partial results.
template <int HD, int QT, int MODE>
__global__ void __launch_bounds__(256, QT == 1 ? 2 : 1) attention_mfma_kernel(AttnArgs a) {
  constexpr bool DEC = MODE == 1, SPLIT = MODE != 0;
  constexpr int KROW = HD * 2;              // bytes per key row
  constexpr int KCH = HD / 8;               // 16-byte chunks per key row
  constexpr int K_BYTES = 64 * KROW;        // 64 keys
  constexpr int V_BYTES = 4 * HD * 32;      // 4 pages of [HD][16]
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int NI = HD / 32;               // direct-to-LDS instructions per wave per operand; also d-tiles
  constexpr int KS = HD / 16;               // MFMA K-steps of the S^T product
  constexpr int BQ = 128 * QT;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // workgroup id -> logical index: each XCD (id % 8) takes a contiguous run of the (beam, kv head, candidate, tile) list
  const int logical = (blockIdx.x & 7) * a.wg_per_xcd + (blockIdx.x >> 3);
  if (logical >= a.total_wg) return;
  const BatchGeom& G = a.g;
  const int g = a.Hq / a.Hkv;
  int rem = logical;
  int split = 0;
  if (SPLIT) { split = rem % a.n_splits; rem /= a.n_splits; }
  const int qt_idx = rem % a.q_tiles; rem /= a.q_tiles;
  int cand = 0;
  if (!DEC) { cand = rem % G.n; rem /= G.n; }
  const int kvh = rem % a.Hkv;
  const int b = rem / a.Hkv;

  // the wavefront index as a scalar: page ids, page bases and LDS destinations then live in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int lq = lane & 31, lh = lane >> 5;
  const int P = G.len_override >= 0 ? G.len_override : G.lens[G.b0 + b];
  const int L = G.L;
  const int cand_idx = b * G.n + cand;
  const size_t m_c0 = (size_t)cand_idx * L;                 // first row of this candidate
  const int rows_total = DEC ? G.n * g : L * g;
  const int r_wg0 = qt_idx * BQ;
  const int32_t* ptab = G.page_table + (size_t)(G.b0 + b) * G.max_pages;

  // --- queries of this wavefront as B-operand fragments (column = query) ---
  int tq[QT];
  bf16x8 qf[QT][KS];
#pragma unroll
  for (int u = 0; u < QT; ++u) {
    int r = r_wg0 + (wave * QT + u) * 32 + lq;
    int rc = r < rows_total ? r : rows_total - 1;
    int t = rc / g, j = rc - t * g;                 // DEC: t is the candidate index within the beam
    tq[u] = t;
    const size_t qrow = DEC ? (size_t)b * G.n + t : m_c0 + t;
    const bf16_t* src = a.q + (qrow * a.Hq + (size_t)kvh * g + j) * HD;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[u][ks] = *(const bf16x8*)(src + ks * 16 + lh * 8);
  }

  floatx16 o[QT][NI];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int u = 0; u < QT; ++u) {
    m_run[u] = -INFINITY;
    l_run[u] = 0.f;
#pragma unroll
    for (int dt = 0; dt < NI; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[u][dt][r] = 0.f;
  }

  const int n_ptiles = (P + 63) >> 6;
  const int n_pages = (P + 15) >> 4;
  int t_hi = (r_wg0 + BQ - 1) / g;
  t_hi = t_hi < L - 1 ? t_hi : L - 1;
  const int n_btiles = DEC ? 0 : ((r_wg0 < rows_total) ? (t_hi >> 6) + 1 : 0);
  // tiles [tile_lo, tile_lo + n_tiles) of the list (prefix tiles, then block tiles)
  const int n_list = n_ptiles + n_btiles;
  const int tile_lo = SPLIT ? (int)((long)split * n_list / a.n_splits) : 0;
  const int n_tiles = SPLIT ? (int)((long)(split + 1) * n_list / a.n_splits) - tile_lo : n_list;

  // one wavefront stages one 16-key group (a page, or 16 block tokens) of the tile: K rows and V^T
  // physical page of this wavefront's 16-key group of a prefix tile (looked up one tile before it is staged, so
  // that the staging loads never wait for the table)
  auto page_of = [&](int tile) {
    int pg = tile * 4 + wave;
    pg = pg < n_pages ? pg : n_pages - 1;
    return tile < n_ptiles ? ptab[pg] : 0;
  };
  auto stage_tile = [&](int tile, int page_id, char* buf) {
    char* kdst = buf + wave * 16 * KROW;
    char* vdst = buf + K_BYTES + wave * HD * 32;
    if (tile < n_ptiles) {
      // scalar page base + a 32-bit lane offset that does not change from tile to tile
      size_t page = (size_t)__builtin_amdgcn_readfirstlane(page_id);
      const bf16_t* ksrc = a.poolK + (page * a.Hkv + kvh) * 16 * HD;
      const bf16_t* vsrc = a.poolV + (page * a.Hkv + kvh) * HD * 16;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        int qi = i * 64 + lane;
        int row = qi / KCH, slot = qi % KCH;
        int chunk = k_swizzle<HD>(wave * 16 + row, slot);
        __builtin_amdgcn_global_load_lds(GLB_PTR(ksrc + (unsigned)(row * HD + chunk * 8)), LDS_PTR(kdst + i * 1024), 16, 0,
                                         0);
      }
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        int qi = i * 64 + lane;
        int d = qi >> 1, half = (qi & 1) ^ ((d >> 3) & 1);       // LDS chunk position qi&1 holds key half `half`
        __builtin_amdgcn_global_load_lds(GLB_PTR(vsrc + (unsigned)(d * 16 + half * 8)), LDS_PTR(vdst + i * 1024), 16, 0, 0);
      }
    } else {
      int key0 = (tile - n_ptiles) * 64 + wave * 16;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        int qi = i * 64 + lane;
        int row = qi / KCH, slot = qi % KCH;
        int chunk = k_swizzle<HD>(wave * 16 + row, slot);
        int key = key0 + row;
        key = key < L ? key : L - 1;
        const bf16_t* src = a.kb + ((m_c0 + key) * a.Hkv + kvh) * HD + chunk * 8;
        __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(kdst + i * 1024), 16, 0, 0);
      }
      const bf16_t* vsrc = a.vbT + ((size_t)cand_idx * a.Hkv + kvh) * HD * a.Lp;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        int qi = i * 64 + lane;
        int d = qi >> 1, half = (qi & 1) ^ ((d >> 3) & 1);
        int key = key0 + half * 8;
        key = key < a.Lp ? key : a.Lp - 8;
        __builtin_amdgcn_global_load_lds(GLB_PTR(vsrc + (size_t)d * a.Lp + key), LDS_PTR(vdst + i * 1024), 16, 0, 0);
      }
    }
  };

  int page_next = 0;
  if (n_tiles > 0) {
    stage_tile(tile_lo, page_of(tile_lo), smem);
    page_next = page_of(tile_lo + 1);
  }
  // pi(i): A-row i of the S^T product carries key pi(i) of the 32-key half tile
  const int pi_row = (lq & 16) | ((lq & 4) << 1) | ((lq & 8) >> 1) | (lq & 3);

  for (int it = 0; it < n_tiles; ++it) {
    const int tile = tile_lo + it;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (it + 1 < n_tiles) {
      stage_tile(tile + 1, page_next, smem + ((it + 1) & 1) * STAGE);
      page_next = page_of(tile + 2);                   // lands while this tile is being multiplied
    }
    const char* Ks = smem + (it & 1) * STAGE;
    const char* Vs = Ks + K_BYTES;
    const bool is_block = tile >= n_ptiles;
    const int key_base = is_block ? (tile - n_ptiles) * 64 : tile * 64;

    // S^T for the two 32-key halves
    floatx16 s[QT][2];
#pragma unroll
    for (int u = 0; u < QT; ++u)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[u][hf][r] = 0.f;
    // K-step outer, key half inner: the two accumulator chains of a query tile alternate. The key fragments are
    // read KPF K-steps ahead of the MFMAs that use them, so that the LDS latency is hidden behind MFMAs.
    constexpr int KPF = 2;
    auto read_kf = [&](int ks, int hf) {
      int row = hf * 32 + pi_row;
      return *(const bf16x8*)(Ks + row * KROW + (k_swizzle<HD>(row, ks * 2 + lh) << 4));
    };
    bf16x8 kf[KPF + 1][2];
#pragma unroll
    for (int ks = 0; ks < KPF; ++ks)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) kf[ks][hf] = read_kf(ks, hf);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * KPF, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + KPF < KS) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) kf[(ks + KPF) % (KPF + 1)][hf] = read_kf(ks + KPF, hf);
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int u = 0; u < QT; ++u)
          s[u][hf] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks % (KPF + 1)][hf], qf[u][ks], s[u][hf], 0, 0, 0);
      if (ks + KPF < KS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * QT, 0);
    }

    // accumulator value r of half hf in this lane is key  key_base + hf*32 + 16*(r/8) + 8*lh + r%8
    bf16x8 pf[QT][4];
#pragma unroll
    for (int u = 0; u < QT; ++u) {
      const bool need_mask = is_block || (key_base + 64 > P);
      if (need_mask) {
        const int limit = is_block ? tq[u] + 1 : P;      // keys < limit are visible
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int key = key_base + hf * 32 + 16 * (r >> 3) + 8 * lh + (r & 7);
            s[u][hf][r] = key < limit ? s[u][hf][r] : -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[u][hf][r]);
      mx = half_wave_max(mx);
      // Reference exponent of the row in the log2 domain (scores are scaled by scale*log2(e) > 0 inside the
      // exponent's FMA). It is always an INTEGER: the weights that multiply V are rounded to bf16, and that rounding
      // commutes with a power-of-two scale, so the rounded operand is the same whichever integer reference a tile
      // happens to see (a streaming evaluation and one that knows the global maximum round the same values). It
      // follows the row maximum lazily: the accumulators are rescaled only when the maximum has grown by more than
      // 2^RESCALE_LOG2 past the reference, so weights reach at most that factor (exact in float; O/l at the end
      // does not depend on the reference) and the 64 multiplications per lane become rare.
      constexpr float RESCALE_LOG2 = 8.f;
      const float m_tile = mx * a.scale_log2e;
      const bool move = m_tile > m_run[u] + RESCALE_LOG2;   // also the first visible key: -inf + 8 = -inf
      if (__any(move)) {
        const float m_new = move ? ceilf(m_tile) : m_run[u];
        const float alpha = move ? __builtin_amdgcn_exp2f(m_run[u] - m_new) : 1.f;   // exp2(-inf) = 0: nothing yet
        l_run[u] *= alpha;
#pragma unroll
        for (int dt = 0; dt < NI; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[u][dt][r] *= alpha;
        m_run[u] = m_new;
      }
      const float m_use = m_run[u] == -INFINITY ? 0.f : m_run[u];   // nothing visible yet: every p below is exp2(-inf) = 0
      float psum = 0.f;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(fmaf(s[u][hf][r], a.scale_log2e, -m_use));
          psum += p;
          pf[u][hf * 2 + (r >> 3)][r & 7] = (bf16_t)p;
        }
      l_run[u] += psum;
    }

    // O^T += V^T P^T : K-step = one 16-key group (page) pg, this lane supplies keys 8*lh .. 8*lh+7 of it
    // (value fragments are read VPF MFMA steps ahead of their use, like the key fragments above)
    constexpr int VPF = 2, NST = 4 * NI;
    auto read_vf = [&](int st) {
      const int pg = st / NI, dt = st % NI;
      return *(const bf16x8*)(Vs + pg * HD * 32 + (dt * 32 + lq) * 32 + ((lh ^ ((lq >> 3) & 1)) << 4));
    };
    bf16x8 vf[VPF + 1];
#pragma unroll
    for (int st = 0; st < VPF; ++st) vf[st] = read_vf(st);
    __builtin_amdgcn_sched_group_barrier(0x100, VPF, 0);
#pragma unroll
    for (int st = 0; st < NST; ++st) {
      const int pg = st / NI, dt = st % NI;
      if (st + VPF < NST) vf[(st + VPF) % (VPF + 1)] = read_vf(st + VPF);
#pragma unroll
      for (int u = 0; u < QT; ++u)
        o[u][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[st % (VPF + 1)], pf[u][pg], o[u][dt], 0, 0, 0);
      if (st + VPF < NST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, QT, 0);
    }
  }

  // normalise and store: lane = query column, accumulator value r of d-tile dt is d = dt*32 + 8*(r/4) + 4*lh + r%4
#pragma unroll
  for (int u = 0; u < QT; ++u) {
    int r = r_wg0 + (wave * QT + u) * 32 + lq;
    float l = half_wave_sum(l_run[u]);
    if (SPLIT) {
      const size_t group = DEC ? (size_t)b * a.Hkv + kvh : ((size_t)b * a.Hkv + kvh) * G.n + cand;
      const size_t prow = ((group * a.q_tiles + qt_idx) * a.n_splits + split) * BQ + (wave * QT + u) * 32 + lq;
      if (lh == 0) { a.part_m[prow] = m_run[u]; a.part_l[prow] = l; }
      float* dst = a.part_o + prow * HD;
#pragma unroll
      for (int dt = 0; dt < NI; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          float4 v = {o[u][dt][r4 * 4], o[u][dt][r4 * 4 + 1], o[u][dt][r4 * 4 + 2], o[u][dt][r4 * 4 + 3]};
          *(float4*)(dst + dt * 32 + 8 * r4 + 4 * lh) = v;
        }
    } else if (r < rows_total) {
      int t = r / g, j = r - t * g;
      float inv = 1.0f / l;
      bf16_t* dst = a.out + ((m_c0 + t) * a.Hq + (size_t)kvh * g + j) * HD;
#pragma unroll
      for (int dt = 0; dt < NI; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          int d = dt * 32 + 8 * r4 + 4 * lh;
#pragma unroll
          for (int e = 0; e < 4; ++e) dst[d + e] = (bf16_t)(o[u][dt][r4 * 4 + e] * inv);
        }
    }
  }
}

template <int HD, int QT, int MODE = 0>
static void launch_attn_variant(const AttnArgs& a, hipStream_t s) {
  constexpr int smem = 2 * (64 * HD * 2 + 4 * HD * 32);
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)attention_mfma_kernel<HD, QT, MODE>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    configured = true;
  }
  attention_mfma_kernel<HD, QT, MODE><<<dim3(a.wg_per_xcd * 8), 256, smem, s>>>(a);
}

// Merge of the partial results of a MODE 2 launch: one wavefront per (row, query head).
template <int HD>
__global__ void __launch_bounds__(64) attention_split_merge_kernel(const float* __restrict__ part_o,
                                                                   const float* __restrict__ part_m,
                                                                   const float* __restrict__ part_l,
                                                                   bf16_t* __restrict__ out, int n, int L, int Hq, int Hkv,
                                                                   int q_tiles, int n_splits) {
  const size_t m = blockIdx.x;
  const int h = blockIdx.y, lane = threadIdx.x;
  const int g = Hq / Hkv, kvh = h / g, j = h - kvh * g;
  const size_t cand_idx = m / L;                           // b*n + i
  const int t = (int)(m - cand_idx * L);
  const int r = t * g + j, qt = r >> 7, rin = r & 127;
  const size_t b = cand_idx / n, i = cand_idx - b * n;
  const size_t group = (b * Hkv + kvh) * n + i;
  const size_t prow0 = (group * q_tiles + qt) * n_splits * 128 + rin;      // + split*128
  float mx = -INFINITY;
  for (int s = 0; s < n_splits; ++s) mx = fmaxf(mx, part_m[prow0 + (size_t)s * 128]);
  float l = 0.f, acc[HD / 64];
#pragma unroll
  for (int u = 0; u < HD / 64; ++u) acc[u] = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const size_t pr = prow0 + (size_t)s * 128;
    const float w = __builtin_amdgcn_exp2f(part_m[pr] - mx);   // 0 for a run that saw no visible key
    l = fmaf(w, part_l[pr], l);
#pragma unroll
    for (int u = 0; u < HD / 64; ++u) acc[u] = fmaf(w, part_o[pr * HD + lane + 64 * u], acc[u]);
  }
  const float inv = 1.0f / l;
#pragma unroll
  for (int u = 0; u < HD / 64; ++u) out[(m * Hq + h) * HD + lane + 64 * u] = (bf16_t)(acc[u] * inv);
}

// Returns false if the shape is not one this kernel takes (head_dim 64/128, 16-token pages).
// part: scratch of part_floats floats for launches whose key tiles are split over several workgroups (may be null).
bool launch_attention_mfma(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* poolK,
                           const bf16_t* poolV, bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp,
                           int max_ctx, float* part, size_t part_floats, hipStream_t s) {
  if ((md.hd != 64 && md.hd != 128) || g.page_tokens != 16 || Lp % 16 != 0) return false;
  AttnArgs a;
  a.q = q; a.kb = kb; a.vbT = vbT; a.poolK = poolK; a.poolV = poolV; a.out = out; a.g = g;
  a.Hq = md.Hq; a.Hkv = md.Hkv; a.Lp = Lp;
  a.n_splits = 1; a.part_o = nullptr; a.part_m = nullptr; a.part_l = nullptr;
  a.scale_log2e = 1.4426950408889634f / sqrtf((float)md.hd);
  int rows = g.L * (md.Hq / md.Hkv);
  // 256-row workgroups only when they waste less padding than 128-row ones (the latter run two per CU)
  int t1 = (rows + 127) / 128, t2 = (rows + 255) / 256;
  bool big = t2 * 256 < t1 * 128;
  a.q_tiles = big ? t2 : t1;
  a.total_wg = g.B * md.Hkv * g.n * a.q_tiles;
  // Few workgroups and a long key list: cut the list into as many runs as still leave all workgroups resident at
  // once (two per CU; one more run would add a second, almost empty round), at least four tiles per run, at most
  // eight runs.
  int list_tiles = (max_ctx + 63) / 64 + (g.L + 63) / 64;
  int splits = 1;
  if (!big && part && a.total_wg < 384 && list_tiles >= 16) {   // short lists: a second kernel costs more than it saves
    splits = 512 / a.total_wg;
    splits = splits > 8 ? 8 : splits;
    splits = splits > list_tiles / 4 ? list_tiles / 4 : splits;
    size_t per_split = (size_t)a.total_wg * 128 * (md.hd + 2);
    if (splits > 1 && (size_t)splits * per_split > part_floats) splits = (int)(part_floats / per_split);
    if (splits < 1) splits = 1;
  }
  if (splits > 1) {
    size_t rows_all = (size_t)a.total_wg * splits * 128;
    a.n_splits = splits;
    a.part_o = part; a.part_m = part + rows_all * md.hd; a.part_l = a.part_m + rows_all;
    a.total_wg *= splits;
    a.wg_per_xcd = (a.total_wg + 7) / 8;
    if (md.hd == 128) launch_attn_variant<128, 1, 2>(a, s); else launch_attn_variant<64, 1, 2>(a, s);
    dim3 grid(g.M, md.Hq);
    if (md.hd == 128)
      attention_split_merge_kernel<128><<<grid, 64, 0, s>>>(a.part_o, a.part_m, a.part_l, out, g.n, g.L, md.Hq, md.Hkv,
                                                           a.q_tiles, splits);
    else
      attention_split_merge_kernel<64><<<grid, 64, 0, s>>>(a.part_o, a.part_m, a.part_l, out, g.n, g.L, md.Hq, md.Hkv,
                                                          a.q_tiles, splits);
    return true;
  }
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  if (md.hd == 128) { if (big) launch_attn_variant<128, 2>(a, s); else launch_attn_variant<128, 1>(a, s); }
  else { if (big) launch_attn_variant<64, 2>(a, s); else launch_attn_variant<64, 1>(a, s); }
  return true;
}

// Prefix part of a single-position launch (g.L == 1): partial results per (beam, kv head, row tile, split).
// q_tiles_out / n_splits_out describe the partial buffers' layout to the merge kernel. part_floats: room in
// `part` (floats); returns false if the shape is not taken or the partials would not fit.
bool launch_attention_mfma_decode_prefix(const bf16_t* q, const bf16_t* poolK, const bf16_t* poolV, const BatchGeom& g,
                                         const ModelDims& md, int max_ctx, float* part, size_t part_floats,
                                         int* q_tiles_out, int* n_splits_out, hipStream_t s) {
  if ((md.hd != 64 && md.hd != 128) || g.page_tokens != 16 || g.L != 1) return false;
  AttnArgs a;
  a.q = q; a.kb = nullptr; a.vbT = nullptr; a.poolK = poolK; a.poolV = poolV; a.out = nullptr; a.g = g;
  a.Hq = md.Hq; a.Hkv = md.Hkv; a.Lp = 16;
  a.scale_log2e = 1.4426950408889634f / sqrtf((float)md.hd);
  int rows = g.n * (md.Hq / md.Hkv);
  a.q_tiles = (rows + 127) / 128;
  int base = g.B * md.Hkv * a.q_tiles;
  int max_tiles = (max_ctx + 63) / 64;
  int splits = (512 + base - 1) / base;                 // about two workgroups per CU ...
  splits = splits > 16 ? 16 : splits;                   // ... but few enough partial results for the merge to stay cheap
  splits = splits > max_tiles ? max_tiles : splits;
  splits = splits < 1 ? 1 : splits;
  size_t per_split = (size_t)base * 128 * (md.hd + 2);
  if (per_split > part_floats) return false;
  if ((size_t)splits * per_split > part_floats) splits = (int)(part_floats / per_split);
  a.n_splits = splits;
  size_t rows_all = (size_t)base * splits * 128;
  a.part_o = part;
  a.part_m = part + rows_all * md.hd;
  a.part_l = a.part_m + rows_all;
  a.total_wg = base * splits;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  if (md.hd == 128) launch_attn_variant<128, 1, 1>(a, s);
  else launch_attn_variant<64, 1, 1>(a, s);
  *q_tiles_out = a.q_tiles;
  *n_splits_out = splits;
  return true;
}
