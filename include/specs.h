/*
 * specs.h - C ABI of the SPECS block-scoring + SubSample hot path for AMD MI355X (gfx950).
 *
 * The paper's SubSample subroutine (Alg. 2) takes a context tr, n draft blocks Y_1..Y_n, the
 * target model, the process reward model and the generator, and selects one block with
 * probability proportional to exp(S_i),
 *     S_i = log(pi_target(Y_i|tr) / pi_gen(Y_i|tr)) + beta * r(Y_i|tr)               (Eq. 1).
 * Producing the three ingredients of S_i is one batched forward pass per model over the L
 * tokens of each block on top of the cached keys/values of tr (Sec. 2 counts the evaluation of a
 * block, i.e. the logits of each of its tokens, as the unit of cost; the appendix on engineering
 * and performance optimisations asks for log-probabilities of the newly generated step only, the
 * prefix being a cache hit). specs_score_blocks is that pass; specs_subsample is the selection.
 *
 * Conventions
 *  - Every tensor pointer is a DEVICE pointer unless the comment says "host". Device memory is
 *    owned by the caller and only borrowed for the duration of the enqueued work.
 *  - All work is enqueued on the stream given to specs_ctx_create; calls return without
 *    synchronising unless stated. The library allocates no device memory: scratch space is
 *    the caller-provided workspace.
 *  - Every call returns a specs_status (0 = OK). Nothing throws or aborts. Conditions only
 *    the device can see (token id out of range, u outside [0,1), non-finite scores) are
 *    recorded in a device status word read back by specs_ctx_status.
 *  - Matrices are row-major [out_features, in_features] (y = x W^T), element type given by
 *    specs_model_desc.dtype (float or bf16). RMSNorm gains are float.
 *  - Rounding (bf16 models): weights, the normalised input of each projection, Q/K/V after
 *    the rotary embedding, the un-normalised softmax weights exp(s - max) that multiply V,
 *    the attention output and the SwiGLU product are bf16; the residual stream, norm
 *    statistics, attention scores, all accumulators, logits, log-sum-exp, token and block
 *    log-probabilities and the reward are float.
 */
#ifndef SPECS_H
#define SPECS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct specs_ctx specs_ctx;
typedef struct specs_model specs_model;
typedef struct specs_prefix specs_prefix;

typedef enum specs_status {
  SPECS_OK = 0,
  SPECS_EINVAL = 1,     /* null pointer, non-positive size, n or L beyond the limits below */
  SPECS_ESHAPE = 2,     /* model description inconsistent (Hq % Hkv, odd head_dim, ...) */
  SPECS_ETOKEN = 3,     /* device: a token id outside [0, vocab); the id is clamped, result undefined */
  SPECS_ERANGE = 4,     /* beta negative or non-finite (host); u outside [0,1) (device) */
  SPECS_ENONFINITE = 5, /* device: NaN/inf score, or every candidate masked; idx = -1 */
  SPECS_EHIP = 6,       /* a HIP runtime call failed */
  SPECS_EWORKSPACE = 7  /* workspace too small for this call */
} specs_status;

enum { SPECS_F32 = 0, SPECS_BF16 = 1 };
enum { SPECS_HEAD_LM = 0, SPECS_HEAD_PRM = 1 };

#define SPECS_GATE_UP_GROUP 32   /* interleave granularity of the fused gate/up matrix */
#define SPECS_MAX_CANDIDATES 1024 /* n limit of specs_subsample */
#define SPECS_MAX_BETAS 64        /* nb limit of specs_subsample */

/* Decoder-only transformer: pre-norm residual blocks, RMSNorm, rotary embedding with
 * rotate-half pairing (i, i + head_dim/2) and absolute 0-based positions, grouped-query
 * attention (query head h reads kv head h / (Hq/Hkv)) with scale 1/sqrt(head_dim), SwiGLU
 * feed-forward, no biases. head = LM: vocabulary projection; PRM: one scalar row. */
typedef struct specs_model_desc {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t dtype;  /* SPECS_F32 | SPECS_BF16: element type of weights, matrix operands and KV cache */
  int32_t head;   /* SPECS_HEAD_LM | SPECS_HEAD_PRM */
  float rope_base, rms_eps;
} specs_model_desc;

typedef struct specs_layer_weights {
  const void* wqkv;    /* [(Hq + 2 Hkv) * hd, d]: q heads, then k heads, then v heads */
  const void* wo;      /* [d, Hq * hd] */
  const void* wgu;     /* [2F, d]: for each group c of 32 FFN units, rows 64c..64c+31 are the gate
                          rows 32c..32c+31 and rows 64c+32..64c+63 the matching up rows (F % 32 == 0) */
  const void* wd;      /* [d, F] */
  const float* g_attn; /* [d] RMSNorm gain before attention */
  const float* g_ffn;  /* [d] RMSNorm gain before the feed-forward */
} specs_layer_weights;

typedef struct specs_weights {
  const void* embed;                  /* [vocab, d] */
  const void* head;                   /* LM: [vocab, d] (untied); PRM: [d] */
  const float* g_final;               /* [d] final RMSNorm gain */
  const specs_layer_weights* layers;  /* HOST array [n_layers] of device pointers (copied by the call) */
} specs_weights;

/* Bytes of workspace that calls with at most max_rows = B*n*L block tokens (or prefill chunk
 * rows) in at most max_blocks = B*n candidate blocks need for this model. Pure host arithmetic. */
size_t specs_workspace_bytes(const specs_model_desc* desc, int64_t max_rows, int32_t max_blocks);

/* Context: device ordinal, a hipStream_t (NULL = the default stream) and the caller's workspace
 * (256-byte aligned). The context keeps no other device memory. */
int specs_ctx_create(int device, void* hip_stream, void* workspace, size_t workspace_bytes, specs_ctx** out);
int specs_ctx_destroy(specs_ctx* ctx);
/* Synchronises the stream, returns the device status word (SPECS_OK or the first device-side
 * error since the last call of this function) in *device_status and clears it. */
int specs_ctx_status(specs_ctx* ctx, int* device_status);

/* Per-kernel timing (HIP events on the context's stream around every launch of the scoring pass, grouped
 * by kernel class). specs_ctx_profile(ctx, 1) clears the records and switches recording on for the calls
 * that follow; specs_ctx_profile_read synchronises the stream and returns, per class, the summed duration
 * in milliseconds and the number of launches since recording was switched on. Recording adds two event
 * records per launch, so leave it off in timed regions. */
enum {
  SPECS_K_QKV = 0,      /* QKV projection */
  SPECS_K_ATTENTION,    /* shared-prefix attention */
  SPECS_K_OPROJ,        /* output projection + residual */
  SPECS_K_GATE_UP,      /* gate/up projection + SiLU*mul */
  SPECS_K_DOWN,         /* down projection + residual */
  SPECS_K_LMHEAD,       /* fused vocabulary head partials */
  SPECS_K_OTHER,        /* embedding, norms, rotary, merges, PRM head */
  SPECS_K_COUNT
};
int specs_ctx_profile(specs_ctx* ctx, int enable);
int specs_ctx_profile_read(specs_ctx* ctx, float* total_ms, int32_t* launches);

/* Wraps the caller's weights (no copy of tensor data; the per-layer pointer table is copied). */
int specs_model_create(specs_ctx* ctx, const specs_model_desc* desc, const specs_weights* w, specs_model** out);
int specs_model_destroy(specs_model* m);

/* The cached trace tr of B independent beams for one model: a paged key/value pool
 *   kv_pool[n_layers][2][num_pages][Hkv][page_tokens * head_dim]   (element type = model dtype), where a
 *   key page-head is [page_tokens][head_dim] (keys stored after the rotary embedding) and a value
 *   page-head is stored transposed, [head_dim][page_tokens], which is the operand order of the
 *   second attention product; the pool must be initialised (no NaN/Inf bit patterns in unused slots),
 * a page table page_table[B][max_pages] of physical page numbers (token j of beam b lives in page
 * page_table[b][j / page_tokens], slot j % page_tokens), the lengths lens[B] (given on host AND on
 * device) and h_last[B][d]: the float residual-stream output of the last layer at the last prefix
 * position, which scores the first token of every candidate block. Wraps caller memory; no copy. */
int specs_prefix_create(specs_ctx* ctx, const specs_model* m, int32_t B, const int32_t* lens_host,
                        int32_t* lens_dev, int32_t page_tokens, void* kv_pool, int64_t num_pages,
                        const int32_t* page_table, int32_t max_pages, float* h_last, specs_prefix** out);
int specs_prefix_destroy(specs_prefix* p);

/* Utility (not part of the timed path): runs the model over the prefix tokens (device, ragged,
 * beams concatenated in order, sum(lens) ids) and fills the key/value pages and h_last. */
int specs_prefill(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* prefix_tokens);

/* Batched verification of the candidate blocks of Alg. 1 step II / Alg. 2: cand[B][n][L] token ids.
 * Every candidate attends to its beam's cached prefix (read once for all n candidates) and
 * causally to its own block. LM head: out[B][n] = log pi(Y_i | tr) = sum over the L tokens of
 * log softmax(z)[y_t], and, if tok_logp != NULL, tok_logp[B][n][L] the per-token terms.
 * PRM head: out[B][n] = sigmoid(w_r . RMSNorm(h)) at the last block token; tok_logp must be NULL.
 * The prefix is not modified. */
int specs_score_blocks(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const int32_t* cand,
                       int32_t n, int32_t L, float* out, float* tok_logp);

/* The two scores the target side contributes to Eq. 1 in one call: logp_target[B][n] = log pi_target(Y_i | tr)
 * and reward[B][n] = r(Y_i | tr) for the same candidate blocks cand[B][n][L], i.e. specs_score_blocks with the
 * target model on its context and with the PRM on its own (Alg. 1 step II evaluates both for every candidate;
 * the two passes are independent and each is enqueued on its context's stream, so with two streams they
 * overlap). tok_logp_target may be NULL. Both prefixes describe the same B traces. Returns the first error. */
int specs_score_target_and_reward(specs_ctx* ctx_target, const specs_model* target, const specs_prefix* p_target,
                                  specs_ctx* ctx_prm, const specs_model* prm, const specs_prefix* p_prm,
                                  const int32_t* cand, int32_t n, int32_t L, float* logp_target,
                                  float* tok_logp_target, float* reward);

/* specs_score_blocks for callers that cannot allocate device memory or hand over a workspace sized for the
 * call: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments,
 * same kernels and bit-identical results, but every working buffer of the pass lives in a scratch array that
 * is part of the library's device image (SPECS_STATIC_SCRATCH_BYTES per GPU, held until the process ends)
 * instead of the context's workspace, which then only has to hold the 256-byte status word. The call
 * allocates nothing and calls no allocating routine. Limits and rules:
 *  - SPECS_EWORKSPACE when specs_workspace_bytes(desc, B*n*L, B*n) exceeds SPECS_STATIC_SCRATCH_BYTES
 *    (the two small benchmark configurations fit; the 1.5B and 7B models do not);
 *  - every call on a GPU shares that GPU's array, whatever the context or stream: calls that overlap on one
 *    GPU race, the caller must order them. Nothing in the array has to start at zero (every buffer is
 *    written before it is read), so the contents a previous call left behind are harmless;
 *  - the block's keys/values are not kept for specs_commit_block: SPECS_EINVAL if it follows this call;
 *  - SPECS_EINVAL while per-kernel timing (specs_ctx_profile) is switched on, since that creates events. */
#define SPECS_STATIC_SCRATCH_BYTES (32u << 20)
int specs_score_blocks_static(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const int32_t* cand,
                              int32_t n, int32_t L, float* out, float* tok_logp);

/* Generation of the candidate blocks (Alg. 1, Step I): the model (LM head) draws n blocks of L tokens
 * for every beam from pi(. | tr), token by token, each token by ancestral sampling from the full
 * softmax at temperature 1: with c_k the running sum of exp(z_v - max z) over ids v <= k,
 * y = min{k : c_k > u * c_limit}, the inverse distribution function in id order read at the caller's
 * uniform u[b][i][t] (device, doubles in [0,1); SPECS_ERANGE on the status word otherwise).
 * vocab_limit: 0, or the number of leading ids that may be drawn (ids >= vocab_limit get probability
 * zero and the rest is renormalised; for models whose vocabulary is larger than that of the models
 * that will score the blocks). Outputs (device): cand[B][n][L] the tokens, logp[B][n] =
 * log pi(Y_i | tr), the block log-likelihood under the law the tokens were drawn from (it comes out of
 * the same pass, so a generator need not be run again as a scorer), and, if tok_logp != NULL,
 * tok_logp[B][n][L] its per-token terms. With vocab_limit < V that law is the restricted softmax,
 * log pi = z_y - logsumexp(z[0..vocab_limit)), whereas specs_score_blocks always scores under the full
 * softmax: use logp as Eq. 1's log pi_gen only together with scores of the same restricted law, or
 * when the log-ratio term vanishes (the target generating, Alg. 1 before the switch); mixing it with
 * full-softmax scores shifts the ratio by log of the probability mass of the permitted ids. The prefix is not modified; the context is left as after
 * specs_score_blocks(cand) with this model and prefix, so specs_commit_block may follow. */
int specs_generate_blocks(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, int32_t n, int32_t L,
                          int32_t vocab_limit, const double* u, int32_t* cand, float* logp, float* tok_logp);

/* Appends candidate `chosen[b]` (host array [B]) of the LAST specs_score_blocks or specs_generate_blocks
 * call made with this model and prefix to the cache (Alg. 1 step II, tr <- (tr, Y)): copies its L keys/values into the
 * pages, sets h_last to its last hidden state and advances lens (host copy inside the handle and
 * the device array). The page table must already cover lens + L tokens. */
int specs_commit_block(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* chosen_host);

/* specs_commit_block with the chosen indices in DEVICE memory (e.g. the idx output of specs_select_and_switch), so
 * that an iteration of Alg. 1 needs no host round trip between selection and commit. An index outside [0, n)
 * (a selection that failed leaves -1 and an error on the status word) is clamped by the kernels. */
int specs_commit_block_dev(specs_ctx* ctx, const specs_model* m, specs_prefix* p, const int32_t* chosen_dev);

/* SubSample (Alg. 2) for B beams and nb inverse temperatures at once:
 *   S_i = logp_target[b][i] - logp_gen[b][i] + beta[j] * reward[b][i]   (Eq. 1; only r is scaled by beta)
 *   w_i = exp(S_i - max S) for live i (mask[b][i] != 0, NULL = all live: Alg. 2's set L = [n])
 *   idx[b][j] = min{k : sum_{i<=k} w_i > u[b][j] * sum_i w_i}, in double precision, index order.
 * beta: host [nb]. u: device double [B][nb], each in [0,1). idx: device int32 [B][nb].
 * max_reward: device float [B] or NULL; max_i reward[b][i] for the switching test of Alg. 1 step III.
 * n <= SPECS_MAX_CANDIDATES, nb <= SPECS_MAX_BETAS. */
int specs_subsample(specs_ctx* ctx, const float* logp_target, const float* logp_gen, const float* reward,
                    const uint8_t* mask, int32_t B, int32_t n, const float* beta, int32_t nb,
                    const double* u, int32_t* idx, float* max_reward);

/* Alg. 1, Steps II (selection) and III (switch) for B beams in one launch. gen_is_draft (device uint8 [B], in/out)
 * says which model generated beam b's candidate blocks: 0 = the target model, so pi_gen = pi_target, the
 * log-ratio of Eq. 1 vanishes and S_i = beta r_i (the collapse to reward-only selection that the paper notes for
 * pi_gen = pi_target; logp_draft[b] is not read); 1 = the draft model, S_i = logp_target - logp_draft + beta r_i.
 * idx[b] is SubSample's choice at the uniform u[b] (Alg. 2, as specs_subsample with nb = 1). Then Step III: a beam
 * with max_i reward[b][i] > tau (strictly) sets its flag, i.e. its blocks come from the draft model from the
 * next iteration on; a set flag is never cleared. max_reward: device [B] or NULL. beta >= 0 finite (SPECS_ERANGE). */
int specs_select_and_switch(specs_ctx* ctx, const float* logp_target, const float* logp_draft, const float* reward,
                            const uint8_t* mask, int32_t B, int32_t n, float beta, float tau, const double* u,
                            uint8_t* gen_is_draft, int32_t* idx, float* max_reward);

/* Which implementation the launches of this process took since the counters were last reset: the matrix-unit
 * (MFMA) kernels, the weight-streaming kernel for at most 32 rows, or the plain kernels that serve the float
 * configuration and shapes the others do not take (K not a multiple of 64, head sizes other than 64/128, pages other
 * than 16 tokens). counts: host int32 [SPECS_PATH_COUNT]; reset != 0 clears the counters after reading them. */
enum {
  SPECS_PATH_GEMM_MFMA = 0,   /* block-tiled MFMA GEMM family */
  SPECS_PATH_GEMM_SKINNY,     /* weight-streaming MFMA GEMM (generation) */
  SPECS_PATH_GEMM_PLAIN,      /* plain GEMM / vocabulary-head kernels */
  SPECS_PATH_ATTN_MFMA,       /* MFMA attention kernels (whole blocks or single positions) */
  SPECS_PATH_ATTN_PLAIN,      /* plain attention kernel */
  SPECS_PATH_COUNT
};
int specs_path_counts(int32_t* counts, int reset);

/* ---- Component entry points -------------------------------------------------------------------
 * The individual contractions of the scoring pass, callable on caller-provided operands so that each
 * kernel can be verified on its own at full benchmark shapes. dtype = SPECS_F32 | SPECS_BF16 is the
 * operand element type; accumulation and outputs are float unless stated. They use the context
 * workspace as scratch (SPECS_EWORKSPACE if it is too small). */

/* C[M][N] = A[M][K] * W[N][K]^T, or C += ... when accumulate != 0 (the residual-stream update). */
int specs_op_linear(specs_ctx* ctx, int32_t dtype, const void* A, const void* W, int32_t M, int32_t N, int32_t K,
                    float* C, int32_t accumulate);
/* act[M][F] (operand dtype) = silu(A Wg^T) * (A Wu^T), Wgu[2F][K] in the interleaved layout of
 * specs_layer_weights.wgu: the SwiGLU feed-forward's first half. */
int specs_op_gate_up(specs_ctx* ctx, int32_t dtype, const void* A, const void* Wgu, int32_t M, int32_t F, int32_t K,
                     void* act);
/* tok_logp[m] = z[tok[m]] - logsumexp_v z[v], z = A[m] . W[v]: the fused vocabulary head. The [M][V]
 * logits are never written to memory. */
int specs_op_lmhead_logprob(specs_ctx* ctx, int32_t dtype, const void* A, const void* W, const int32_t* tok,
                            int32_t M, int32_t V, int32_t K, float* tok_logp);
/* Shared-prefix attention of one layer: q[B*n*L][Hq][hd], block keys/values kb, vb[B*n*L][Hkv][hd]
 * (all operand dtype, after the rotary embedding), prefix keys/values of `layer` from the handle's
 * pages; out[B*n*L][Hq*hd] (operand dtype). */
int specs_op_attention(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, int32_t layer, const void* q,
                       const void* kb, const void* vb, int32_t n, int32_t L, void* out);

/* The QKV projection of one layer with what the pass does to its result: q, k rotated by the rotary
 * embedding at absolute position lens[b] + t (pairs (i, i + hd/2), base from the model description), all
 * three converted to the operand dtype. A[B*n*L][d] (operand dtype) is the normalised layer input,
 * Wqkv[(Hq+2Hkv)*hd][d] the layer's projection. Outputs (operand dtype): q[B*n*L][Hq][hd],
 * kblk[B*n*L][Hkv][hd] and the values transposed per candidate, vT[B*n][Hkv][hd][Lp] with Lp = L rounded
 * up to 16 and the padding zeroed: the layouts specs_op_attention's kernels read. Runs the kernels the pass
 * runs for this shape (bf16 with more than 32 rows: the rotary embedding in the GEMM epilogue). */
int specs_op_qkv_rope(specs_ctx* ctx, const specs_model* m, const specs_prefix* p, const void* A, const void* Wqkv,
                      int32_t n, int32_t L, void* q, void* kblk, void* vT);

const char* specs_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPECS_H */
