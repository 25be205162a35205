// Host side of the C ABI: handle bookkeeping, argument checks, workspace carving and the order
// in which the kernels of one scoring pass are enqueued. No device memory is allocated here.
#include "common.h"
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#define HIP_TRY(expr)                    \
  do {                                   \
    hipError_t e_ = (expr);              \
    if (e_ != hipSuccess) return SPECS_EHIP; \
  } while (0)

// Scratch of specs_score_blocks_static: callers that may not allocate (code under graph capture, tight serving
// loops) get the pass's working buffers from this array instead of a workspace. Every GPU the library runs on
// holds its own copy at its own address; in host code the name is only a handle for hipGetSymbolAddress, so the
// address is looked up once per device (specs_ctx_create, with that device current) and kept in
// g_static_scratch, which is what kernels and carve() are given.
static __device__ __align__(256) unsigned char scratch[SPECS_STATIC_SCRATCH_BYTES];
enum { kMaxDevices = 64 };
static char* g_static_scratch[kMaxDevices];
static std::mutex g_static_scratch_mutex;

static int resolve_static_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return SPECS_OK;      // such a context has no static scratch
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (g_static_scratch[device]) return SPECS_OK;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SPECS_EHIP;
  g_static_scratch[device] = (char*)ptr;
  return SPECS_OK;
}

static std::atomic<int> g_path_counts[SPECS_PATH_COUNT];
void count_path(int which) {
  if (which >= 0 && which < SPECS_PATH_COUNT) g_path_counts[which].fetch_add(1, std::memory_order_relaxed);
}
extern "C" int specs_path_counts(int32_t* counts, int reset) {
  if (!counts) return SPECS_EINVAL;
  for (int i = 0; i < SPECS_PATH_COUNT; ++i)
    counts[i] = reset ? g_path_counts[i].exchange(0, std::memory_order_relaxed)
                      : g_path_counts[i].load(std::memory_order_relaxed);
  return SPECS_OK;
}

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline size_t esize(int dtype) { return dtype == SPECS_BF16 ? 2 : 4; }

struct specs_model {
  specs_model_desc desc;
  specs_weights w;
  std::vector<specs_layer_weights> layers;
};

struct specs_prefix {
  const specs_model* model;
  int B, page_tokens, max_pages;
  int64_t num_pages;
  std::vector<int32_t> lens;
  int32_t* lens_dev;
  char* kv_pool;
  const int32_t* page_table;
  float* h_last;
};

// Carved view of the workspace for one (model, rows) pair. Offsets are recomputed per call;
// nothing but the status word persists between calls except the block keys/values and the
// final residual stream, which specs_commit_block reads.
struct Workspace {
  int* status;
  float* x;          // [R, d] residual stream (float)
  char* a;           // [R, max(d, Hq*hd)] operand of the next projection (T)
  float* qkv;        // [R, (Hq+2Hkv)*hd]
  char* q;           // [R, Hq*hd] (T)
  char* attn;        // [R, Hq*hd] (T)
  char* kblk;        // [n_layers][R, Hkv*hd] (T)
  char* vblk;        // [n_layers][C, Hkv*hd, Lp] transposed block values
  float* gu;         // [R, 2F]
  char* act;         // [R, F] (T)
  float* cs;         // [R, hd] cos | sin
  float* part_max;   // [R, tiles]
  float* part_sum;
  float* zt;         // [R]
  float* tokl;       // [R] per-token log-probs when the caller passes no buffer
  int32_t* chosen;   // [B]
  float* xs;         // [C, d] residual stream of one position per block (generation steps; the PRM's last layer)
  float* logits;     // [C, V] next-token logits of a generation step (LM heads)
  char* sample;      // per-chunk softmax statistics of the sampling kernels (LM heads)
  size_t total;
};

static inline int round16(int v) { return (v + 15) & ~15; }

// R rows in C = B*n candidate blocks. Block values are kept transposed with the block length padded
// to a multiple of 16, hence up to R + 16*C value columns per layer.
static Workspace carve(char* base, const specs_model_desc& d, int64_t R, int64_t C) {
  Workspace w;
  size_t off = 0, es = esize(d.dtype);
  auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += align256(bytes); return p; };
  size_t qd = (size_t)d.n_q_heads * d.head_dim, kvd = (size_t)d.n_kv_heads * d.head_dim;
  size_t wide = qd > (size_t)d.d_model ? qd : (size_t)d.d_model;
  w.status = (int*)take(256);
  w.x = (float*)take(R * d.d_model * 4);
  w.a = take(R * wide * es);
  w.qkv = (float*)take(R * (qd + 2 * kvd) * 4);
  w.q = take(R * qd * es);
  w.attn = take(R * qd * es);
  w.kblk = take((size_t)d.n_layers * R * kvd * es);
  w.vblk = take((size_t)d.n_layers * (R + 16 * C) * kvd * es);
  w.gu = (float*)take(R * 2 * (size_t)d.ffn * 4);
  w.act = take(R * (size_t)d.ffn * es);
  w.cs = (float*)take(R * d.head_dim * 4);
  size_t tiles = d.head == SPECS_HEAD_LM ? (size_t)lmhead_simple_tiles(d.vocab) : 1;
  w.part_max = (float*)take(R * tiles * 4);
  w.part_sum = (float*)take(R * tiles * 4);
  w.zt = (float*)take(R * 4);
  w.tokl = (float*)take(R * 4);
  w.chosen = (int32_t*)take((size_t)(C > 0 ? C : 1) * 4);
  bool lm = d.head == SPECS_HEAD_LM;
  w.xs = (float*)take((size_t)C * d.d_model * 4);
  w.logits = (float*)take(lm ? (size_t)C * d.vocab * 4 : 0);
  w.sample = take(lm ? sample_scratch_bytes((int)C) : 0);
  w.total = off;
  return w;
}

struct KernelProfile {
  bool on = false;
  std::vector<hipEvent_t> pool;
  size_t used = 0;
  struct Rec { int cls; hipEvent_t a, b; };
  std::vector<Rec> recs;
  hipEvent_t get() {
    if (used == pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[used++];
  }
};

struct specs_ctx {
  KernelProfile prof;
  int device;
  hipStream_t stream;
  char* workspace;
  size_t workspace_bytes;
  // what the last specs_score_blocks left in the workspace (for specs_commit_block)
  const specs_model* last_model;
  const specs_prefix* last_prefix;
  int last_n, last_L;
};

static bool desc_ok(const specs_model_desc& d) {
  if (d.n_layers <= 0 || d.d_model <= 0 || d.n_q_heads <= 0 || d.n_kv_heads <= 0 || d.head_dim <= 0 || d.ffn <= 0 ||
      d.vocab <= 0)
    return false;
  if (d.n_q_heads % d.n_kv_heads) return false;
  if (d.head_dim % 2) return false;
  if (d.ffn % SPECS_GATE_UP_GROUP) return false;
  if (d.dtype != SPECS_F32 && d.dtype != SPECS_BF16) return false;
  if (d.head != SPECS_HEAD_LM && d.head != SPECS_HEAD_PRM) return false;
  if (!(d.rope_base > 0.f) || !(d.rms_eps >= 0.f)) return false;
  return true;
}

extern "C" size_t specs_workspace_bytes(const specs_model_desc* desc, int64_t max_rows, int32_t max_blocks) {
  if (!desc || max_rows <= 0 || max_blocks <= 0 || !desc_ok(*desc)) return 0;
  return carve(nullptr, *desc, max_rows, max_blocks).total;
}

extern "C" int specs_ctx_create(int device, void* hip_stream, void* workspace, size_t workspace_bytes, specs_ctx** out) {
  if (!out || !workspace || workspace_bytes < 256 || ((uintptr_t)workspace & 255)) return SPECS_EINVAL;
  HIP_TRY(hipSetDevice(device));
  if (int rc = resolve_static_scratch(device)) return rc;
  specs_ctx* c = new (std::nothrow) specs_ctx();
  if (!c) return SPECS_EINVAL;
  c->device = device;
  c->stream = (hipStream_t)hip_stream;
  c->workspace = (char*)workspace;
  c->workspace_bytes = workspace_bytes;
  c->last_model = nullptr;
  c->last_prefix = nullptr;
  c->last_n = c->last_L = 0;
  hipError_t e = hipMemsetAsync(workspace, 0, 256, c->stream);   // the status word
  if (e != hipSuccess) { delete c; return SPECS_EHIP; }
  *out = c;
  return SPECS_OK;
}

extern "C" int specs_ctx_destroy(specs_ctx* ctx) {
  if (ctx)
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
  delete ctx;
  return SPECS_OK;
}

extern "C" int specs_ctx_profile(specs_ctx* ctx, int enable) {
  if (!ctx) return SPECS_EINVAL;
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  ctx->prof.on = enable != 0;
  ctx->prof.used = 0;
  ctx->prof.recs.clear();
  return SPECS_OK;
}

extern "C" int specs_ctx_profile_read(specs_ctx* ctx, float* total_ms, int32_t* launches) {
  if (!ctx || !total_ms || !launches) return SPECS_EINVAL;
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  for (int c = 0; c < SPECS_K_COUNT; ++c) { total_ms[c] = 0.f; launches[c] = 0; }
  for (const KernelProfile::Rec& r : ctx->prof.recs) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
    total_ms[r.cls] += ms;
    launches[r.cls] += 1;
  }
  return SPECS_OK;
}

// Runs `stmt` (kernel launches on stream s), bracketed by events of class `cls` when profiling is on.
#define PROFILED(ctx, cls, s, stmt)                                   \
  do {                                                                \
    if ((ctx)->prof.on) {                                             \
      hipEvent_t e0_ = (ctx)->prof.get(), e1_ = (ctx)->prof.get();    \
      if (e0_ && e1_) {                                               \
        (void)hipEventRecord(e0_, s);                                 \
        stmt;                                                         \
        (void)hipEventRecord(e1_, s);                                 \
        (ctx)->prof.recs.push_back({cls, e0_, e1_});                  \
      } else { stmt; }                                                \
    } else { stmt; }                                                  \
  } while (0)

extern "C" int specs_ctx_status(specs_ctx* ctx, int* device_status) {
  if (!ctx || !device_status) return SPECS_EINVAL;
  int v = 0;
  HIP_TRY(hipMemcpyAsync(&v, ctx->workspace, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  if (v != 0) {
    HIP_TRY(hipMemsetAsync(ctx->workspace, 0, sizeof(int), ctx->stream));
    HIP_TRY(hipStreamSynchronize(ctx->stream));
  }
  *device_status = v;
  return SPECS_OK;
}

extern "C" int specs_model_create(specs_ctx* ctx, const specs_model_desc* desc, const specs_weights* w, specs_model** out) {
  if (!ctx || !desc || !w || !out) return SPECS_EINVAL;
  if (!desc_ok(*desc)) return SPECS_ESHAPE;
  if (!w->embed || !w->head || !w->g_final || !w->layers) return SPECS_EINVAL;
  for (int l = 0; l < desc->n_layers; ++l) {
    const specs_layer_weights& L = w->layers[l];
    if (!L.wqkv || !L.wo || !L.wgu || !L.wd || !L.g_attn || !L.g_ffn) return SPECS_EINVAL;
  }
  specs_model* m = new (std::nothrow) specs_model();
  if (!m) return SPECS_EINVAL;
  m->desc = *desc;
  m->w = *w;
  m->layers.assign(w->layers, w->layers + desc->n_layers);
  m->w.layers = m->layers.data();
  *out = m;
  return SPECS_OK;
}

extern "C" int specs_model_destroy(specs_model* m) {
  delete m;
  return SPECS_OK;
}

extern "C" int specs_prefix_create(specs_ctx* ctx, const specs_model* m, int32_t B, const int32_t* lens_host,
                                   int32_t* lens_dev, int32_t page_tokens, void* kv_pool, int64_t num_pages,
                                   const int32_t* page_table, int32_t max_pages, float* h_last, specs_prefix** out) {
  if (!ctx || !m || !lens_host || !lens_dev || !kv_pool || !page_table || !h_last || !out) return SPECS_EINVAL;
  if (B <= 0 || page_tokens <= 0 || num_pages <= 0 || max_pages <= 0) return SPECS_EINVAL;
  for (int b = 0; b < B; ++b) {
    if (lens_host[b] < 0) return SPECS_EINVAL;
    if ((int64_t)lens_host[b] > (int64_t)max_pages * page_tokens) return SPECS_EINVAL;
  }
  specs_prefix* p = new (std::nothrow) specs_prefix();
  if (!p) return SPECS_EINVAL;
  p->model = m;
  p->B = B;
  p->page_tokens = page_tokens;
  p->max_pages = max_pages;
  p->num_pages = num_pages;
  p->lens.assign(lens_host, lens_host + B);
  p->lens_dev = lens_dev;
  p->kv_pool = (char*)kv_pool;
  p->page_table = page_table;
  p->h_last = h_last;
  *out = p;
  return SPECS_OK;
}

extern "C" int specs_prefix_destroy(specs_prefix* p) {
  delete p;
  return SPECS_OK;
}

// ---------------------------------------------------------------------------------------------
template <typename T>
static T* pool_ptr(const specs_prefix* p, const specs_model_desc& d, int layer, int which) {
  size_t per = (size_t)p->num_pages * d.n_kv_heads * p->page_tokens * d.head_dim;
  return (T*)p->kv_pool + ((size_t)layer * 2 + which) * per;
}

// Geometry of a launch that covers whole blocks: rows m = (b*n + i)*L + t over all beams of the prefix handle.
static BatchGeom block_geom(const specs_prefix* p, int n, int L) {
  BatchGeom g;
  g.B = p->B; g.n = n; g.L = L; g.M = p->B * n * L; g.b0 = 0; g.len_override = -1; g.t0 = 0; g.Lk = L;
  g.lens = p->lens_dev; g.page_table = p->page_table; g.max_pages = p->max_pages; g.page_tokens = p->page_tokens;
  return g;
}

static ModelDims dims_of(const specs_model_desc& d) {
  ModelDims md;
  md.d = d.d_model; md.Hq = d.n_q_heads; md.Hkv = d.n_kv_heads; md.hd = d.head_dim; md.F = d.ffn; md.V = d.vocab;
  md.eps = d.rms_eps; md.rope_base = d.rope_base;
  return md;
}

template <typename T>
static void gemm(const T* A, const T* W, float* C, int M, int N, int K, GemmEpilogue epi, hipStream_t s) {
  count_path(SPECS_PATH_GEMM_PLAIN);
  launch_gemm_simple<T>(A, W, C, M, N, K, epi, s);
}
template <>
void gemm<bf16_t>(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, GemmEpilogue epi, hipStream_t s) {
  int e = epi == EPI_RESIDUAL_ADD ? MFMA_RESIDUAL : MFMA_STORE;
  if (launch_gemm_mfma(e, A, W, M, N, K, C, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 0, s)) {
    count_path(SPECS_PATH_GEMM_MFMA);
  } else {
    count_path(SPECS_PATH_GEMM_PLAIN);
    launch_gemm_simple<bf16_t>(A, W, C, M, N, K, epi, s);
  }
}

// K-split form of x += A W^T for the residual projections: when the plan says that slicing K fills the CUs
// better, writes the partial products to `part` (room for max_split of them) and returns their number;
// the caller's next normalisation kernel sums them into x. Returns 0 when the product was added to x directly.
template <typename T>
static int gemm_residual_split(const T* A, const T* W, float* x, float* part, int max_split, int M, int N, int K,
                               hipStream_t s) {
  gemm<T>(A, W, x, M, N, K, EPI_RESIDUAL_ADD, s);
  return 0;
}
template <>
int gemm_residual_split<bf16_t>(const bf16_t* A, const bf16_t* W, float* x, float* part, int max_split, int M, int N,
                                int K, hipStream_t s) {
  if (M <= 32 && max_split >= 1) {                       // a few rows: stream the weights once, K in slices
    int sp = skinny_gemm_split(N, K, max_split);
    if (launch_gemm_skinny(MFMA_STORE, A, W, M, N, K, part, nullptr, sp, s)) { count_path(SPECS_PATH_GEMM_SKINNY); return sp; }
  }
  // Also with one slice the product goes to `part` and the normalisation kernel, which reads x anyway, adds it:
  // the GEMM's epilogue then only writes, instead of waiting for a read of x before every store.
  int bm = 0, split = 1;
  if (K % 64 == 0 && max_split > 1) mfma_gemm_plan(M, N, K, max_split, &bm, &split);
  if (max_split >= 1 &&
      launch_gemm_mfma(MFMA_STORE, A, W, M, N, K, part, nullptr, nullptr, nullptr, nullptr, nullptr, split, bm, s)) {
    count_path(SPECS_PATH_GEMM_MFMA);
    return split;
  }
  gemm<bf16_t>(A, W, x, M, N, K, EPI_RESIDUAL_ADD, s);
  return 0;
}

// C = A W^T as up to max_split K slices [slices][M][N] that the consumer adds up; returns their number.
template <typename T>
static int gemm_store_split(const T* A, const T* W, float* C, int max_split, int M, int N, int K, hipStream_t s) {
  gemm<T>(A, W, C, M, N, K, EPI_STORE_F32, s);
  return 1;
}
template <>
int gemm_store_split<bf16_t>(const bf16_t* A, const bf16_t* W, float* C, int max_split, int M, int N, int K,
                             hipStream_t s) {
  if (M <= 32 && max_split >= 1) {
    int sp = skinny_gemm_split(N, K, max_split);
    if (launch_gemm_skinny(MFMA_STORE, A, W, M, N, K, C, nullptr, sp, s)) { count_path(SPECS_PATH_GEMM_SKINNY); return sp; }
  }
  gemm<bf16_t>(A, W, C, M, N, K, EPI_STORE_F32, s);
  return 1;
}

template <typename T>
static bool qkv_rope_fused(const T*, const T*, const float*, T*, T*, T*, const BatchGeom&, const ModelDims&, int,
                           hipStream_t) {
  return false;
}
template <>
bool qkv_rope_fused<bf16_t>(const bf16_t* A, const bf16_t* W, const float* cs, bf16_t* q, bf16_t* kb, bf16_t* vT,
                            const BatchGeom& g, const ModelDims& md, int Lp, hipStream_t s) {
  if (!launch_gemm_mfma_qkv_rope(A, W, cs, q, kb, vT, g, md, Lp, s)) return false;
  count_path(SPECS_PATH_GEMM_MFMA);
  return true;
}

// act[M,F] = silu(A Wg^T) * (A Wu^T) with Wgu interleaved by 32 rows
template <typename T>
static void gate_up(const T* A, const T* Wgu, float* gu, T* act, int M, int F, int K, hipStream_t s) {
  count_path(SPECS_PATH_GEMM_PLAIN);
  launch_gemm_simple<T>(A, Wgu, gu, M, 2 * F, K, EPI_STORE_F32, s);
  launch_silu_mul<T>(gu, act, M, F, s);
}
template <>
void gate_up<bf16_t>(const bf16_t* A, const bf16_t* Wgu, float* gu, bf16_t* act, int M, int F, int K, hipStream_t s) {
  if (M <= 32 && launch_gemm_skinny(MFMA_SWIGLU, A, Wgu, M, 2 * F, K, nullptr, act, 1, s)) { count_path(SPECS_PATH_GEMM_SKINNY); return; }
  if (launch_gemm_mfma(MFMA_SWIGLU, A, Wgu, M, 2 * F, K, nullptr, act, nullptr, nullptr, nullptr, nullptr, 1, 0, s)) {
    count_path(SPECS_PATH_GEMM_MFMA);
    return;
  }
  count_path(SPECS_PATH_GEMM_PLAIN);
  launch_gemm_simple<bf16_t>(A, Wgu, gu, M, 2 * F, K, EPI_STORE_F32, s);
  launch_silu_mul<bf16_t>(gu, act, M, F, s);
}

// per-(row, column tile) log-sum-exp partials + target logit; returns the number of column tiles
template <typename T>
static int lmhead_partials(const T* A, const T* W, const int32_t* tok, float* pm, float* ps, float* zt, int M, int V,
                           int K, hipStream_t s) {
  int tiles = 0;
  count_path(SPECS_PATH_GEMM_PLAIN);
  launch_lmhead_partials_simple<T>(A, W, tok, pm, ps, zt, M, V, K, &tiles, s);
  return tiles;
}
template <>
int lmhead_partials<bf16_t>(const bf16_t* A, const bf16_t* W, const int32_t* tok, float* pm, float* ps, float* zt, int M,
                            int V, int K, hipStream_t s) {
  if (launch_gemm_mfma(MFMA_LMHEAD, A, W, M, V, K, nullptr, nullptr, tok, pm, ps, zt, 1, 0, s)) {
    count_path(SPECS_PATH_GEMM_MFMA);
    return mfma_lmhead_tiles(V);
  }
  count_path(SPECS_PATH_GEMM_PLAIN);
  int tiles = 0;
  launch_lmhead_partials_simple<bf16_t>(A, W, tok, pm, ps, zt, M, V, K, &tiles, s);
  return tiles;
}

// scratch: floats free for the duration of the call (partial results of single-position launches)
template <typename T>
static void attention(const T* q, const T* kb, const T* vbT, const T* pK, const T* pV, T* out, const BatchGeom& g,
                      const ModelDims& md, int Lp, int max_ctx, float* scratch, size_t scratch_floats, hipStream_t s);

// The trunk over g.M rows: every row attends to its beam's cached prefix and causally to the earlier
// positions of its own block. Row m embeds tokens[m * tok_stride]. Leaves the final residual stream in x and the
// per-layer block keys/values in ws.kblk / ws.vblk (laid out for blocks of g.Lk tokens; a launch with g.L = 1 and
// g.t0 = t adds position t of every block). commit_pages: also write them into the prefix pages (prefill).
// last_token_only (whole-block launches): the caller reads x only at the last token of every block (the PRM head),
// so after the last layer's keys and values exist for all rows, its attention output, O projection and
// feed-forward run for that one row per block; the other rows of x are left as the last layer found them.
template <typename T>
static void run_trunk(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const Workspace& ws,
                      const BatchGeom& g, float* x, const int32_t* tokens, int tok_stride, int max_ctx,
                      bool commit_pages, int64_t R, int64_t C, hipStream_t s, bool last_token_only = false) {
  const specs_model_desc& d = m->desc;
  ModelDims md = dims_of(d);
  const int Lp = round16(g.Lk);
  int qd = md.Hq * md.hd, kvd = md.Hkv * md.hd;
  PROFILED(ctx, SPECS_K_OTHER, s,
           launch_embed<T>(tokens, tok_stride, (const T*)m->w.embed, x, g.M, md.d, md.V, ws.status, s);
           launch_rope_table(ws.cs, g, md.hd, md.rope_base, s));
  // ws.gu ([R, 2F] floats) is free while the residual projections run (the fused gate/up kernel never writes
  // it, the unfused path has consumed it by then), so it holds their K-split partial products.
  const int max_split = (int)((2 * (size_t)md.F) / (size_t)md.d);
  bool normed = false;                                   // ws.a already holds RMSNorm(x) * g_attn of this layer
  for (int l = 0; l < d.n_layers; ++l) {
    const specs_layer_weights& L = m->layers[l];
    T* kb = (T*)ws.kblk + (size_t)l * R * kvd;
    T* vb = (T*)ws.vblk + (size_t)l * (R + 16 * C) * kvd;
    T* pK = pool_ptr<T>(p, d, l, 0);
    T* pV = pool_ptr<T>(p, d, l, 1);
    if (!normed) PROFILED(ctx, SPECS_K_OTHER, s, launch_rmsnorm<T>(x, L.g_attn, (T*)ws.a, g.M, md.d, md.eps, s));
    // whole-block bf16 launches: rotary embedding, conversion and value transposition inside the projection's epilogue
    bool fused_rope = false;
    if (g.M > 32)
      PROFILED(ctx, SPECS_K_QKV, s,
               fused_rope = qkv_rope_fused<T>((const T*)ws.a, (const T*)L.wqkv, ws.cs, (T*)ws.q, kb, vb, g, md, Lp, s));
    if (!fused_rope) {
      int qkv_parts = 1;                                 // ws.qkv has room for R / g.M slices of the projection
      PROFILED(ctx, SPECS_K_QKV, s,
               qkv_parts = gemm_store_split<T>((const T*)ws.a, (const T*)L.wqkv, ws.qkv, (int)(R / g.M < 8 ? R / g.M : 8),
                                               g.M, qd + 2 * kvd, md.d, s));
      PROFILED(ctx, SPECS_K_OTHER, s, launch_rope_split<T>(ws.qkv, qkv_parts, ws.cs, (T*)ws.q, kb, vb, g, Lp, md, s));
    }
    if (last_token_only && l == d.n_layers - 1 && g.L > 1 && g.t0 == 0 && !commit_pages) {
      BatchGeom gl = g;                                  // one row per block: its last position
      gl.L = 1; gl.M = (int)C; gl.t0 = g.L - 1; gl.Lk = g.L;
      T* q1 = (T*)ws.a;                                  // the projection has consumed ws.a
      PROFILED(ctx, SPECS_K_OTHER, s,
               launch_gather_last_rows<T>((const T*)ws.q, q1, (int)C, g.L, qd, s);
               launch_gather_last_rows<float>(x, ws.xs, (int)C, g.L, md.d, s));
      PROFILED(ctx, SPECS_K_ATTENTION, s,
               attention<T>(q1, kb, vb, pK, pV, (T*)ws.attn, gl, md, Lp, max_ctx, ws.gu, (size_t)R * 2 * md.F, s));
      int pl = 0;
      PROFILED(ctx, SPECS_K_OPROJ, s,
               pl = gemm_residual_split<T>((const T*)ws.attn, (const T*)L.wo, ws.xs, ws.gu, max_split, gl.M, md.d, qd, s));
      if (pl)
        PROFILED(ctx, SPECS_K_OTHER, s,
                 launch_add_partials_rmsnorm<T>(ws.xs, ws.gu, pl, 0, L.g_ffn, (T*)ws.a, gl.M, md.d, md.eps, s));
      else
        PROFILED(ctx, SPECS_K_OTHER, s, launch_rmsnorm<T>(ws.xs, L.g_ffn, (T*)ws.a, gl.M, md.d, md.eps, s));
      PROFILED(ctx, SPECS_K_GATE_UP, s,
               gate_up<T>((const T*)ws.a, (const T*)L.wgu, ws.gu, (T*)ws.act, gl.M, md.F, md.d, s));
      PROFILED(ctx, SPECS_K_DOWN, s,
               pl = gemm_residual_split<T>((const T*)ws.act, (const T*)L.wd, ws.xs, ws.gu, max_split, gl.M, md.d, md.F, s));
      if (pl)
        PROFILED(ctx, SPECS_K_OTHER, s,
                 launch_add_partials_rmsnorm<T>(ws.xs, ws.gu, pl, 0, nullptr, (T*)ws.a, gl.M, md.d, md.eps, s));
      PROFILED(ctx, SPECS_K_OTHER, s, launch_scatter_last_rows(ws.xs, x, (int)C, g.L, md.d, s));
      break;
    }
    PROFILED(ctx, SPECS_K_ATTENTION, s,
             attention<T>((const T*)ws.q, kb, vb, pK, pV, (T*)ws.attn, g, md, Lp, max_ctx, ws.gu,
                          (size_t)R * 2 * md.F, s));
    if (commit_pages) launch_kv_commit<T>(kb, vb, pK, pV, g, md, Lp, nullptr, s);
    int parts = 0;
    PROFILED(ctx, SPECS_K_OPROJ, s,
             parts = gemm_residual_split<T>((const T*)ws.attn, (const T*)L.wo, x, ws.gu, max_split, g.M, md.d, qd, s));
    if (parts)
      PROFILED(ctx, SPECS_K_OTHER, s,
               launch_add_partials_rmsnorm<T>(x, ws.gu, parts, 0, L.g_ffn, (T*)ws.a, g.M, md.d, md.eps, s));
    else
      PROFILED(ctx, SPECS_K_OTHER, s, launch_rmsnorm<T>(x, L.g_ffn, (T*)ws.a, g.M, md.d, md.eps, s));
    PROFILED(ctx, SPECS_K_GATE_UP, s,
             gate_up<T>((const T*)ws.a, (const T*)L.wgu, ws.gu, (T*)ws.act, g.M, md.F, md.d, s));
    PROFILED(ctx, SPECS_K_DOWN, s,
             parts = gemm_residual_split<T>((const T*)ws.act, (const T*)L.wd, x, ws.gu, max_split, g.M, md.d, md.F, s));
    normed = false;
    if (parts) {
      // the sum of the partials is folded into the next layer's first normalisation (none after the last layer)
      const float* next_gain = l + 1 < d.n_layers ? m->layers[l + 1].g_attn : nullptr;
      PROFILED(ctx, SPECS_K_OTHER, s,
               launch_add_partials_rmsnorm<T>(x, ws.gu, parts, 0, next_gain, (T*)ws.a, g.M, md.d, md.eps, s));
      normed = next_gain != nullptr;
    }
  }
}

// base / bytes: where the pass's buffers live (the context's workspace, or the static scratch of this device).
// The status word is the context's in both cases.
template <typename T>
static int score_impl(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const int32_t* cand, int n, int L,
                      float* out, float* tok_logp, char* base, size_t bytes) {
  const specs_model_desc& d = m->desc;
  int64_t R = (int64_t)p->B * n * L;
  int64_t C = (int64_t)p->B * n;
  Workspace ws = carve(base, d, R, C);
  if (ws.total > bytes) return SPECS_EWORKSPACE;
  ws.status = (int*)ctx->workspace;
  BatchGeom g = block_geom(p, n, L);
  int max_ctx = 0;
  for (int b = 0; b < p->B; ++b) max_ctx = p->lens[b] > max_ctx ? p->lens[b] : max_ctx;
  hipStream_t s = ctx->stream;
  run_trunk<T>(ctx, m, p, ws, g, ws.x, cand, 1, max_ctx, false, R, C, s, d.head == SPECS_HEAD_PRM);
  if (d.head == SPECS_HEAD_LM) {
    int tiles = 0;
    PROFILED(ctx, SPECS_K_OTHER, s,
             launch_rmsnorm_shifted<T>(ws.x, p->h_last, m->w.g_final, (T*)ws.a, g, d.d_model, d.rms_eps, s));
    PROFILED(ctx, SPECS_K_LMHEAD, s,
             tiles = lmhead_partials<T>((const T*)ws.a, (const T*)m->w.head, cand, ws.part_max, ws.part_sum, ws.zt,
                                        g.M, d.vocab, d.d_model, s));
    PROFILED(ctx, SPECS_K_OTHER, s,
             launch_lmhead_merge(ws.part_max, ws.part_sum, ws.zt, tiles, tok_logp, ws.tokl, out, g, s));
  } else {
    PROFILED(ctx, SPECS_K_OTHER, s,
             launch_prm_head<T>(ws.x, m->w.g_final, (const T*)m->w.head, out, g, d.d_model, d.rms_eps, s));
  }
  HIP_TRY(hipGetLastError());
  bool in_workspace = base == ctx->workspace;        // only then can specs_commit_block find the block's keys/values
  ctx->last_model = in_workspace ? m : nullptr;
  ctx->last_prefix = in_workspace ? p : nullptr;
  ctx->last_n = n;
  ctx->last_L = L;
  return SPECS_OK;
}

static int score_args_ok(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const int32_t* cand, int32_t n,
                         int32_t L, float* out, float* tok_logp) {
  if (!ctx || !m || !p || !cand || !out) return SPECS_EINVAL;
  if (p->model != m) return SPECS_EINVAL;
  if (n <= 0 || L <= 0) return SPECS_EINVAL;
  if (m->desc.head == SPECS_HEAD_PRM && tok_logp) return SPECS_EINVAL;
  if ((int64_t)p->B * n * L > (int64_t)1 << 30) return SPECS_EINVAL;
  for (int b = 0; b < p->B; ++b)
    if (p->lens[b] < 1) return SPECS_EINVAL;       // the first block token is scored from the last prefix position
  return SPECS_OK;
}

extern "C" int specs_score_blocks(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const int32_t* cand,
                                  int32_t n, int32_t L, float* out, float* tok_logp) {
  if (int rc = score_args_ok(ctx, m, p, cand, n, L, out, tok_logp)) return rc;
  HIP_TRY(hipSetDevice(ctx->device));
  return m->desc.dtype == SPECS_BF16
             ? score_impl<bf16_t>(ctx, m, p, cand, n, L, out, tok_logp, ctx->workspace, ctx->workspace_bytes)
             : score_impl<float>(ctx, m, p, cand, n, L, out, tok_logp, ctx->workspace, ctx->workspace_bytes);
}

extern "C" int specs_score_target_and_reward(specs_ctx* ctx_target, const specs_model* target,
                                             const specs_prefix* p_target, specs_ctx* ctx_prm, const specs_model* prm,
                                             const specs_prefix* p_prm, const int32_t* cand, int32_t n, int32_t L,
                                             float* logp_target, float* tok_logp_target, float* reward) {
  if (!target || !prm || target->desc.head != SPECS_HEAD_LM || prm->desc.head != SPECS_HEAD_PRM) return SPECS_EINVAL;
  if (!p_target || !p_prm || p_target->B != p_prm->B) return SPECS_EINVAL;
  if (int rc = score_args_ok(ctx_target, target, p_target, cand, n, L, logp_target, tok_logp_target)) return rc;
  if (int rc = score_args_ok(ctx_prm, prm, p_prm, cand, n, L, reward, nullptr)) return rc;
  if (int rc = specs_score_blocks(ctx_target, target, p_target, cand, n, L, logp_target, tok_logp_target)) return rc;
  return specs_score_blocks(ctx_prm, prm, p_prm, cand, n, L, reward, nullptr);
}

extern "C" int specs_score_blocks_static(specs_ctx* ctx, const specs_model* m, const specs_prefix* p,
                                         const int32_t* cand, int32_t n, int32_t L, float* out, float* tok_logp) {
  if (int rc = score_args_ok(ctx, m, p, cand, n, L, out, tok_logp)) return rc;
  if (ctx->device < 0 || ctx->device >= kMaxDevices || !g_static_scratch[ctx->device]) return SPECS_EINVAL;
  if (ctx->prof.on) return SPECS_EINVAL;             // per-kernel timing creates events: not in this entry point
  HIP_TRY(hipSetDevice(ctx->device));
  char* base = g_static_scratch[ctx->device];        // the device address, never the array's name
  return m->desc.dtype == SPECS_BF16
             ? score_impl<bf16_t>(ctx, m, p, cand, n, L, out, tok_logp, base, SPECS_STATIC_SCRATCH_BYTES)
             : score_impl<float>(ctx, m, p, cand, n, L, out, tok_logp, base, SPECS_STATIC_SCRATCH_BYTES);
}

// Alg. 1, Step I: n blocks of L tokens per beam, one position at a time. Step t: next-token logits from the
// state that precedes position t (the prefix's last hidden state for t = 0), one token per candidate by inverse
// CDF from u, then that token goes through the trunk at position t, which adds its keys/values to the block
// buffers. After the last step the workspace holds what specs_score_blocks(cand) would have left there.
template <typename T>
static int generate_impl(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, int n, int L, int limit,
                         const double* u, int32_t* cand, float* out, float* tok_logp) {
  const specs_model_desc& d = m->desc;
  int64_t R = (int64_t)p->B * n * L;
  int64_t C = (int64_t)p->B * n;
  Workspace ws = carve(ctx->workspace, d, R, C);
  if (ws.total > ctx->workspace_bytes) return SPECS_EWORKSPACE;
  BatchGeom g = block_geom(p, n, 1);                   // one row per candidate
  g.Lk = L;
  int max_ctx = 0;
  for (int b = 0; b < p->B; ++b) max_ctx = p->lens[b] > max_ctx ? p->lens[b] : max_ctx;
  hipStream_t s = ctx->stream;
  float* tl = tok_logp ? tok_logp : ws.tokl;
  launch_broadcast_hlast(p->h_last, ws.xs, g, d.d_model, s);
  for (int t = 0; t < L; ++t) {
    g.t0 = t;
    PROFILED(ctx, SPECS_K_OTHER, s, launch_rmsnorm<T>(ws.xs, m->w.g_final, (T*)ws.a, g.M, d.d_model, d.rms_eps, s));
    PROFILED(ctx, SPECS_K_LMHEAD, s,
             gemm_store_split<T>((const T*)ws.a, (const T*)m->w.head, ws.logits, 1, g.M, d.vocab, d.d_model, s));
    PROFILED(ctx, SPECS_K_OTHER, s,
             launch_sample_tokens(ws.logits, g.M, d.vocab, limit, u, cand, tl, L, t, ws.sample, ws.status, s));
    run_trunk<T>(ctx, m, p, ws, g, ws.xs, cand + t, L, max_ctx, false, R, C, s);
  }
  launch_scatter_last_rows(ws.xs, ws.x, (int)C, L, d.d_model, s);
  launch_block_sum(tl, out, L, (int)C, s);
  HIP_TRY(hipGetLastError());
  ctx->last_model = m;
  ctx->last_prefix = p;
  ctx->last_n = n;
  ctx->last_L = L;
  return SPECS_OK;
}

extern "C" int specs_generate_blocks(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, int32_t n, int32_t L,
                                     int32_t vocab_limit, const double* u, int32_t* cand, float* logp,
                                     float* tok_logp) {
  if (!ctx || !m || !p || !u || !cand || !logp) return SPECS_EINVAL;
  if (p->model != m || m->desc.head != SPECS_HEAD_LM) return SPECS_EINVAL;
  if (n <= 0 || L <= 0 || vocab_limit < 0 || vocab_limit > m->desc.vocab) return SPECS_EINVAL;
  if ((int64_t)p->B * n * L > (int64_t)1 << 30) return SPECS_EINVAL;
  for (int b = 0; b < p->B; ++b)
    if (p->lens[b] < 1) return SPECS_EINVAL;           // the first token is drawn from the last prefix position
  HIP_TRY(hipSetDevice(ctx->device));
  int limit = vocab_limit ? vocab_limit : m->desc.vocab;
  return m->desc.dtype == SPECS_BF16 ? generate_impl<bf16_t>(ctx, m, p, n, L, limit, u, cand, logp, tok_logp)
                                     : generate_impl<float>(ctx, m, p, n, L, limit, u, cand, logp, tok_logp);
}

template <typename T>
static int prefill_impl(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* tokens) {
  const specs_model_desc& d = m->desc;
  // largest chunk the workspace can hold
  int64_t maxlen = 0;
  for (int b = 0; b < p->B; ++b) maxlen = p->lens[b] > maxlen ? p->lens[b] : maxlen;
  int64_t R = maxlen < 2048 ? maxlen : 2048;
  while (R > 0 && carve(nullptr, d, R, 1).total > ctx->workspace_bytes) R /= 2;
  if (R <= 0) return SPECS_EWORKSPACE;
  Workspace ws = carve(ctx->workspace, d, R, 1);
  hipStream_t s = ctx->stream;
  int64_t off = 0;
  for (int b = 0; b < p->B; ++b) {
    int len = p->lens[b];
    for (int c0 = 0; c0 < len; c0 += (int)R) {
      int rows = len - c0 < R ? len - c0 : (int)R;
      BatchGeom g = block_geom(p, 1, rows);
      g.B = 1; g.M = rows; g.b0 = b; g.len_override = c0;
      run_trunk<T>(ctx, m, p, ws, g, ws.x, tokens + off + c0, 1, c0, true, R, 1, s);
      if (c0 + rows == len) launch_copy_rows(ws.x, p->h_last, g, d.d_model, nullptr, s);
    }
    off += len;
  }
  HIP_TRY(hipGetLastError());
  ctx->last_model = nullptr;
  ctx->last_prefix = nullptr;
  return SPECS_OK;
}

extern "C" int specs_prefill(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* prefix_tokens) {
  if (!ctx || !m || !p || !prefix_tokens) return SPECS_EINVAL;
  if (p->model != m) return SPECS_EINVAL;
  HIP_TRY(hipSetDevice(ctx->device));
  return m->desc.dtype == SPECS_BF16 ? prefill_impl<bf16_t>(ctx, m, p, prefix_tokens)
                                     : prefill_impl<float>(ctx, m, p, prefix_tokens);
}

__global__ void advance_lens_kernel(int32_t* lens, int B, int L) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) lens[b] += L;
}

// chosen_dev != nullptr: the indices are already in device memory (no copy, no host-side range check)
template <typename T>
static int commit_impl(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* chosen_host,
                       const int32_t* chosen_dev = nullptr) {
  const specs_model_desc& d = m->desc;
  int n = ctx->last_n, L = ctx->last_L;
  int64_t R = (int64_t)p->B * n * L, C = (int64_t)p->B * n;
  Workspace ws = carve(ctx->workspace, d, R, C);
  ModelDims md = dims_of(d);
  hipStream_t s = ctx->stream;
  const int32_t* chosen = chosen_dev;
  if (!chosen) {
    HIP_TRY(hipMemcpyAsync(ws.chosen, chosen_host, sizeof(int32_t) * p->B, hipMemcpyHostToDevice, s));
    chosen = ws.chosen;
  }
  BatchGeom g = block_geom(p, n, L);
  size_t kvd = (size_t)md.Hkv * md.hd;
  for (int l = 0; l < d.n_layers; ++l)
    launch_kv_commit<T>((const T*)ws.kblk + (size_t)l * R * kvd, (const T*)ws.vblk + (size_t)l * (R + 16 * C) * kvd,
                        pool_ptr<T>(p, d, l, 0), pool_ptr<T>(p, d, l, 1), g, md, round16(L), chosen, s);
  launch_copy_rows(ws.x, p->h_last, g, d.d_model, chosen, s);
  advance_lens_kernel<<<(p->B + 63) / 64, 64, 0, s>>>(p->lens_dev, p->B, L);
  HIP_TRY(hipGetLastError());
  for (int b = 0; b < p->B; ++b) p->lens[b] += L;
  ctx->last_model = nullptr;
  ctx->last_prefix = nullptr;
  return SPECS_OK;
}

extern "C" int specs_commit_block(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* chosen_host) {
  if (!ctx || !m || !p || !chosen_host) return SPECS_EINVAL;
  if (ctx->last_model != m || ctx->last_prefix != p || ctx->last_L <= 0) return SPECS_EINVAL;
  for (int b = 0; b < p->B; ++b) {
    if (chosen_host[b] < 0 || chosen_host[b] >= ctx->last_n) return SPECS_EINVAL;
    if ((int64_t)p->lens[b] + ctx->last_L > (int64_t)p->max_pages * p->page_tokens) return SPECS_EINVAL;
  }
  HIP_TRY(hipSetDevice(ctx->device));
  return m->desc.dtype == SPECS_BF16 ? commit_impl<bf16_t>(ctx, m, p, chosen_host)
                                     : commit_impl<float>(ctx, m, p, chosen_host);
}

extern "C" int specs_commit_block_dev(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* chosen_dev) {
  if (!ctx || !m || !p || !chosen_dev) return SPECS_EINVAL;
  if (ctx->last_model != m || ctx->last_prefix != p || ctx->last_L <= 0) return SPECS_EINVAL;
  for (int b = 0; b < p->B; ++b)
    if ((int64_t)p->lens[b] + ctx->last_L > (int64_t)p->max_pages * p->page_tokens) return SPECS_EINVAL;
  HIP_TRY(hipSetDevice(ctx->device));
  return m->desc.dtype == SPECS_BF16 ? commit_impl<bf16_t>(ctx, m, p, nullptr, chosen_dev)
                                     : commit_impl<float>(ctx, m, p, nullptr, chosen_dev);
}

extern "C" int specs_subsample(specs_ctx* ctx, const float* logp_target, const float* logp_gen, const float* reward,
                               const uint8_t* mask, int32_t B, int32_t n, const float* beta, int32_t nb,
                               const double* u, int32_t* idx, float* max_reward) {
  if (!ctx || !logp_target || !logp_gen || !reward || !beta || !u || !idx) return SPECS_EINVAL;
  if (B <= 0 || n <= 0 || nb <= 0 || n > SPECS_MAX_CANDIDATES || nb > SPECS_MAX_BETAS) return SPECS_EINVAL;
  for (int j = 0; j < nb; ++j)
    if (!std::isfinite(beta[j]) || beta[j] < 0.f) return SPECS_ERANGE;
  HIP_TRY(hipSetDevice(ctx->device));
  launch_subsample(logp_target, logp_gen, reward, mask, B, n, beta, nb, u, idx, max_reward, nullptr, 0.f,
                   (int*)ctx->workspace, ctx->stream);
  HIP_TRY(hipGetLastError());
  return SPECS_OK;
}

extern "C" int specs_select_and_switch(specs_ctx* ctx, const float* logp_target, const float* logp_draft,
                                       const float* reward, const uint8_t* mask, int32_t B, int32_t n, float beta,
                                       float tau, const double* u, uint8_t* gen_is_draft, int32_t* idx,
                                       float* max_reward) {
  if (!ctx || !logp_target || !logp_draft || !reward || !u || !gen_is_draft || !idx) return SPECS_EINVAL;
  if (B <= 0 || n <= 0 || n > SPECS_MAX_CANDIDATES) return SPECS_EINVAL;
  if (!std::isfinite(beta) || beta < 0.f || std::isnan(tau)) return SPECS_ERANGE;
  HIP_TRY(hipSetDevice(ctx->device));
  launch_subsample(logp_target, logp_draft, reward, mask, B, n, &beta, 1, u, idx, max_reward, gen_is_draft, tau,
                   (int*)ctx->workspace, ctx->stream);
  HIP_TRY(hipGetLastError());
  return SPECS_OK;
}

// ---------------------------------------------------------------- component entry points
extern "C" int specs_op_linear(specs_ctx* ctx, int32_t dtype, const void* A, const void* W, int32_t M, int32_t N,
                               int32_t K, float* C, int32_t accumulate) {
  if (!ctx || !A || !W || !C || M <= 0 || N <= 0 || K <= 0) return SPECS_EINVAL;
  if (dtype != SPECS_F32 && dtype != SPECS_BF16) return SPECS_EINVAL;
  HIP_TRY(hipSetDevice(ctx->device));
  GemmEpilogue e = accumulate ? EPI_RESIDUAL_ADD : EPI_STORE_F32;
  if (dtype == SPECS_BF16) {
    // same K-split decision as inside the scoring pass, as far as the workspace has room for the partial products
    size_t per = (size_t)M * N * sizeof(float);
    size_t room = ctx->workspace_bytes > 256 ? (ctx->workspace_bytes - 256) / per : 0;
    int bm = 0, split = 1;
    if (K % 64 == 0 && room > 1) mfma_gemm_plan(M, N, K, room > 8 ? 8 : (int)room, &bm, &split);
    float* part = (float*)(ctx->workspace + 256);
    int sk = M <= 32 && room >= 1 ? skinny_gemm_split(N, K, room > 8 ? 8 : (int)room) : 0;
    if (sk && launch_gemm_skinny(MFMA_STORE, (const bf16_t*)A, (const bf16_t*)W, M, N, K, part, nullptr, sk,
                                 ctx->stream)) {
      launch_add_partials_rmsnorm<bf16_t>(C, part, sk, accumulate ? 0 : 1, nullptr, nullptr, M, N, 0.f, ctx->stream);
      ctx->last_model = nullptr;
    } else if (split > 1 && launch_gemm_mfma(MFMA_STORE, (const bf16_t*)A, (const bf16_t*)W, M, N, K, part, nullptr, nullptr,
                                      nullptr, nullptr, nullptr, split, bm, ctx->stream)) {
      launch_add_partials_rmsnorm<bf16_t>(C, part, split, accumulate ? 0 : 1, nullptr, nullptr, M, N, 0.f, ctx->stream);
      ctx->last_model = nullptr;                         // the workspace no longer holds a scored block
    } else {
      gemm<bf16_t>((const bf16_t*)A, (const bf16_t*)W, C, M, N, K, e, ctx->stream);
    }
  } else {
    gemm<float>((const float*)A, (const float*)W, C, M, N, K, e, ctx->stream);
  }
  HIP_TRY(hipGetLastError());
  return SPECS_OK;
}

extern "C" int specs_op_gate_up(specs_ctx* ctx, int32_t dtype, const void* A, const void* Wgu, int32_t M, int32_t F,
                                int32_t K, void* act) {
  if (!ctx || !A || !Wgu || !act || M <= 0 || F <= 0 || K <= 0 || F % SPECS_GATE_UP_GROUP) return SPECS_EINVAL;
  if (dtype != SPECS_F32 && dtype != SPECS_BF16) return SPECS_EINVAL;
  size_t need = 256 + align256((size_t)M * 2 * F * 4);
  if (need > ctx->workspace_bytes) return SPECS_EWORKSPACE;
  float* gu = (float*)(ctx->workspace + 256);
  HIP_TRY(hipSetDevice(ctx->device));
  if (dtype == SPECS_BF16) gate_up<bf16_t>((const bf16_t*)A, (const bf16_t*)Wgu, gu, (bf16_t*)act, M, F, K, ctx->stream);
  else gate_up<float>((const float*)A, (const float*)Wgu, gu, (float*)act, M, F, K, ctx->stream);
  HIP_TRY(hipGetLastError());
  ctx->last_model = nullptr;
  return SPECS_OK;
}

extern "C" int specs_op_lmhead_logprob(specs_ctx* ctx, int32_t dtype, const void* A, const void* W, const int32_t* tok,
                                       int32_t M, int32_t V, int32_t K, float* tok_logp) {
  if (!ctx || !A || !W || !tok || !tok_logp || M <= 0 || V <= 0 || K <= 0) return SPECS_EINVAL;
  if (dtype != SPECS_F32 && dtype != SPECS_BF16) return SPECS_EINVAL;
  size_t tiles = (size_t)lmhead_simple_tiles(V);
  size_t per = align256((size_t)M * tiles * 4);
  if (256 + 2 * per + 2 * align256((size_t)M * 4) > ctx->workspace_bytes) return SPECS_EWORKSPACE;
  float* pm = (float*)(ctx->workspace + 256);
  float* ps = (float*)(ctx->workspace + 256 + per);
  float* zt = (float*)(ctx->workspace + 256 + 2 * per);
  float* tl = (float*)(ctx->workspace + 256 + 2 * per + align256((size_t)M * 4));
  HIP_TRY(hipSetDevice(ctx->device));
  int nt = dtype == SPECS_BF16
               ? lmhead_partials<bf16_t>((const bf16_t*)A, (const bf16_t*)W, tok, pm, ps, zt, M, V, K, ctx->stream)
               : lmhead_partials<float>((const float*)A, (const float*)W, tok, pm, ps, zt, M, V, K, ctx->stream);
  BatchGeom g = {};
  g.B = 1; g.n = M; g.L = 1; g.M = M; g.Lk = 1;
  launch_lmhead_merge(pm, ps, zt, nt, nullptr, tl, tok_logp, g, ctx->stream);
  HIP_TRY(hipGetLastError());
  ctx->last_model = nullptr;
  return SPECS_OK;
}

template <typename T>
static void attention(const T* q, const T* kb, const T* vbT, const T* pK, const T* pV, T* out, const BatchGeom& g,
                      const ModelDims& md, int Lp, int max_ctx, float* scratch, size_t scratch_floats, hipStream_t s) {
  count_path(SPECS_PATH_ATTN_PLAIN);
  launch_attention_simple<T>(q, kb, vbT, pK, pV, out, g, md, Lp, max_ctx, s);
}
template <>
void attention<bf16_t>(const bf16_t* q, const bf16_t* kb, const bf16_t* vbT, const bf16_t* pK, const bf16_t* pV,
                       bf16_t* out, const BatchGeom& g, const ModelDims& md, int Lp, int max_ctx, float* scratch,
                       size_t scratch_floats, hipStream_t s) {
  bool whole_blocks = g.t0 == 0 && g.Lk == g.L;
  // Launches with at least ~160 workgroups of 256 stacked rows take the two-phase kernel (measured 3-8 % faster
  // at the 7B shapes); smaller ones the one-phase kernel, which cuts long key lists over several workgroups.
  const long stacked = (long)g.B * md.Hkv * (((long)g.n * g.L * (md.Hq / md.Hkv) + 255) / 256);
  if (whole_blocks) {
    if (stacked >= 160 && launch_attention_pingpong(q, kb, vbT, pK, pV, out, g, md, Lp, max_ctx, nullptr, 0, s)) {
      count_path(SPECS_PATH_ATTN_MFMA);
      return;
    }
    if (launch_attention_mfma(q, kb, vbT, pK, pV, out, g, md, Lp, max_ctx, scratch, scratch_floats, s)) {
      count_path(SPECS_PATH_ATTN_MFMA);
      return;
    }
  } else if (g.L == 1 && scratch &&
             launch_attention_decode(q, kb, vbT, pK, pV, out, g, md, Lp, max_ctx, scratch, scratch_floats, s)) {
    count_path(SPECS_PATH_ATTN_MFMA);
    return;
  }
  count_path(SPECS_PATH_ATTN_PLAIN);
  launch_attention_simple<bf16_t>(q, kb, vbT, pK, pV, out, g, md, Lp, max_ctx, s);
}

extern "C" int specs_op_attention(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, int32_t layer,
                                  const void* q, const void* kb, const void* vb, int32_t n, int32_t L, void* out) {
  if (!ctx || !m || !p || !q || !kb || !vb || !out || n <= 0 || L <= 0) return SPECS_EINVAL;
  if (p->model != m || layer < 0 || layer >= m->desc.n_layers) return SPECS_EINVAL;
  const specs_model_desc& d = m->desc;
  BatchGeom g = block_geom(p, n, L);
  int max_ctx = 0;
  for (int b = 0; b < p->B; ++b) max_ctx = p->lens[b] > max_ctx ? p->lens[b] : max_ctx;
  ModelDims md = dims_of(d);
  const int Lp = round16(L), cands = p->B * n;
  size_t vt_bytes = (size_t)cands * md.Hkv * md.hd * Lp * esize(d.dtype);
  if (256 + align256(vt_bytes) > ctx->workspace_bytes) return SPECS_EWORKSPACE;
  char* vT = ctx->workspace + 256;
  HIP_TRY(hipSetDevice(ctx->device));
  if (d.dtype == SPECS_BF16) {
    launch_transpose_v<bf16_t>((const bf16_t*)vb, (bf16_t*)vT, cands, md.Hkv, md.hd, L, Lp, ctx->stream);
    attention<bf16_t>((const bf16_t*)q, (const bf16_t*)kb, (const bf16_t*)vT, pool_ptr<bf16_t>(p, d, layer, 0),
                      pool_ptr<bf16_t>(p, d, layer, 1), (bf16_t*)out, g, md, Lp, max_ctx, nullptr, 0, ctx->stream);
  } else {
    launch_transpose_v<float>((const float*)vb, (float*)vT, cands, md.Hkv, md.hd, L, Lp, ctx->stream);
    attention<float>((const float*)q, (const float*)kb, (const float*)vT, pool_ptr<float>(p, d, layer, 0),
                     pool_ptr<float>(p, d, layer, 1), (float*)out, g, md, Lp, max_ctx, nullptr, 0, ctx->stream);
  }
  HIP_TRY(hipGetLastError());
  ctx->last_model = nullptr;
  return SPECS_OK;
}

extern "C" int specs_op_qkv_rope(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const void* A,
                                 const void* Wqkv, int32_t n, int32_t L, void* q, void* kblk, void* vT) {
  if (!ctx || !m || !p || !A || !Wqkv || !q || !kblk || !vT || n <= 0 || L <= 0) return SPECS_EINVAL;
  if (p->model != m || (int64_t)p->B * n * L > (int64_t)1 << 30) return SPECS_EINVAL;
  const specs_model_desc& d = m->desc;
  BatchGeom g = block_geom(p, n, L);
  ModelDims md = dims_of(d);
  const int Lp = round16(L);
  const size_t width = (size_t)(md.Hq + 2 * md.Hkv) * md.hd;
  const size_t cs_bytes = align256((size_t)g.M * md.hd * sizeof(float));
  const size_t qkv_bytes = align256((size_t)g.M * width * sizeof(float));
  if (256 + cs_bytes + qkv_bytes > ctx->workspace_bytes) return SPECS_EWORKSPACE;
  float* cs = (float*)(ctx->workspace + 256);
  float* qkv = (float*)(ctx->workspace + 256 + cs_bytes);
  hipStream_t s = ctx->stream;
  HIP_TRY(hipSetDevice(ctx->device));
  launch_rope_table(cs, g, md.hd, md.rope_base, s);
  if (d.dtype == SPECS_BF16) {
    bool fused = g.M > 32 && qkv_rope_fused<bf16_t>((const bf16_t*)A, (const bf16_t*)Wqkv, cs, (bf16_t*)q, (bf16_t*)kblk,
                                                    (bf16_t*)vT, g, md, Lp, s);
    if (!fused) {
      int parts = gemm_store_split<bf16_t>((const bf16_t*)A, (const bf16_t*)Wqkv, qkv, 1, g.M, (int)width, md.d, s);
      launch_rope_split<bf16_t>(qkv, parts, cs, (bf16_t*)q, (bf16_t*)kblk, (bf16_t*)vT, g, Lp, md, s);
    }
  } else {
    int parts = gemm_store_split<float>((const float*)A, (const float*)Wqkv, qkv, 1, g.M, (int)width, md.d, s);
    launch_rope_split<float>(qkv, parts, cs, (float*)q, (float*)kblk, (float*)vT, g, Lp, md, s);
  }
  HIP_TRY(hipGetLastError());
  ctx->last_model = nullptr;
  return SPECS_OK;
}

extern "C" const char* specs_strerror(int status) {
  switch (status) {
    case SPECS_OK: return "ok";
    case SPECS_EINVAL: return "invalid argument";
    case SPECS_ESHAPE: return "inconsistent model description";
    case SPECS_ETOKEN: return "token id outside the vocabulary";
    case SPECS_ERANGE: return "beta or uniform outside its range";
    case SPECS_ENONFINITE: return "non-finite score or no live candidate";
    case SPECS_EHIP: return "HIP runtime error";
    case SPECS_EWORKSPACE: return "workspace too small";
    default: return "unknown status";
  }
}
