"""ctypes binding of include/specs.h: same names, torch tensors in place of raw pointers.

Argument marshalling only. Tensors must already live on the GPU (the library borrows their
memory); handles are opaque ctypes pointers.
"""
import ctypes as C
import os

_LIB = None
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecs_hip.so")

EXPORTED_SYMBOLS = [
    "specs_workspace_bytes", "specs_ctx_create", "specs_ctx_destroy", "specs_ctx_status", "specs_model_create",
    "specs_model_destroy", "specs_prefix_create", "specs_prefix_destroy", "specs_prefill", "specs_score_blocks",
    "specs_commit_block", "specs_subsample", "specs_strerror", "specs_generate_blocks",
    "specs_op_linear", "specs_op_gate_up", "specs_op_lmhead_logprob", "specs_op_attention",
    "specs_ctx_profile", "specs_ctx_profile_read", "specs_score_blocks_static", "specs_score_target_and_reward", "specs_op_qkv_rope",
    "specs_commit_block_dev", "specs_select_and_switch", "specs_path_counts",
]
PATH_CLASSES = ("gemm_mfma", "gemm_skinny", "gemm_plain", "attn_mfma", "attn_plain")
KERNEL_CLASSES = ("qkv", "attention", "oproj", "gate_up", "down", "lmhead", "other")

SPECS_F32, SPECS_BF16 = 0, 1
SPECS_HEAD_LM, SPECS_HEAD_PRM = 0, 1
GATE_UP_GROUP = 32


class SpecsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = _LIB.specs_strerror(code).decode() if _LIB is not None else "?"
        super().__init__(f"{where}: status {code} ({msg})")


class ModelDescC(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                         "dtype", "head")] + [("rope_base", C.c_float), ("rms_eps", C.c_float)]


class LayerWeightsC(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("wqkv", "wo", "wgu", "wd", "g_attn", "g_ffn")]


class WeightsC(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("head", C.c_void_p), ("g_final", C.c_void_p),
                ("layers", C.POINTER(LayerWeightsC))]


def load_library():
    """Load libspecs_hip.so (built by __graft_entry__.build()). Raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: run `python __graft_entry__.py` (build()) first; "
                           "there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.specs_workspace_bytes.restype = C.c_size_t
    lib.specs_workspace_bytes.argtypes = [C.POINTER(ModelDescC), i64, i32]
    lib.specs_ctx_create.argtypes = [C.c_int, vp, vp, C.c_size_t, C.POINTER(vp)]
    lib.specs_ctx_destroy.argtypes = [vp]
    lib.specs_ctx_status.argtypes = [vp, C.POINTER(C.c_int)]
    lib.specs_model_create.argtypes = [vp, C.POINTER(ModelDescC), C.POINTER(WeightsC), C.POINTER(vp)]
    lib.specs_model_destroy.argtypes = [vp]
    lib.specs_prefix_create.argtypes = [vp, vp, i32, C.POINTER(i32), vp, i32, vp, i64, vp, i32, vp, C.POINTER(vp)]
    lib.specs_prefix_destroy.argtypes = [vp]
    lib.specs_prefill.argtypes = [vp, vp, vp, vp]
    lib.specs_score_blocks.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp]
    lib.specs_score_blocks_static.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp]
    lib.specs_score_target_and_reward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.specs_generate_blocks.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.specs_commit_block.argtypes = [vp, vp, vp, C.POINTER(i32)]
    lib.specs_commit_block_dev.argtypes = [vp, vp, vp, vp]
    lib.specs_select_and_switch.argtypes = [vp, vp, vp, vp, vp, i32, i32, C.c_float, C.c_float, vp, vp, vp, vp]
    lib.specs_path_counts.argtypes = [C.POINTER(i32), C.c_int]
    lib.specs_subsample.argtypes = [vp, vp, vp, vp, vp, i32, i32, C.POINTER(C.c_float), i32, vp, vp, vp]
    lib.specs_ctx_profile.argtypes = [vp, C.c_int]
    lib.specs_ctx_profile_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32)]
    lib.specs_op_linear.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp, i32]
    lib.specs_op_gate_up.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp]
    lib.specs_op_lmhead_logprob.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, vp]
    lib.specs_op_attention.argtypes = [vp, vp, vp, i32, vp, vp, vp, i32, i32, vp]
    lib.specs_op_qkv_rope.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.specs_strerror.restype = C.c_char_p
    lib.specs_strerror.argtypes = [C.c_int]
    for name in EXPORTED_SYMBOLS:
        if name not in ("specs_workspace_bytes", "specs_strerror"):
            getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


def _check(code, where):
    if code != 0:
        raise SpecsError(code, where)


def _ptr(t, dtype=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise ValueError("tensor required")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def make_desc(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab, dtype, head, rope_base=10000.0,
              rms_eps=1e-6):
    return ModelDescC(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
                      SPECS_BF16 if dtype == "bf16" else SPECS_F32,
                      SPECS_HEAD_PRM if head == "prm" else SPECS_HEAD_LM, rope_base, rms_eps)


def specs_workspace_bytes(desc, max_rows, max_B):
    return load_library().specs_workspace_bytes(C.byref(desc), max_rows, max_B)


def specs_ctx_create(device_index, stream_handle, workspace):
    import torch
    lib = load_library()
    out = C.c_void_p()
    assert workspace.dtype == torch.uint8
    _check(lib.specs_ctx_create(device_index, C.c_void_p(stream_handle), _ptr(workspace), workspace.numel(),
                                C.byref(out)), "specs_ctx_create")
    return out


def specs_ctx_destroy(ctx):
    _check(load_library().specs_ctx_destroy(ctx), "specs_ctx_destroy")


def specs_ctx_status(ctx):
    v = C.c_int(0)
    _check(load_library().specs_ctx_status(ctx, C.byref(v)), "specs_ctx_status")
    return v.value


def specs_ctx_profile(ctx, enable):
    _check(load_library().specs_ctx_profile(ctx, 1 if enable else 0), "specs_ctx_profile")


def specs_ctx_profile_read(ctx):
    """{kernel class: (total ms, launches)} since profiling was switched on."""
    n = len(KERNEL_CLASSES)
    ms, cnt = (C.c_float * n)(), (C.c_int32 * n)()
    _check(load_library().specs_ctx_profile_read(ctx, ms, cnt), "specs_ctx_profile_read")
    return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}


def specs_model_create(ctx, desc, embed, head, g_final, layers):
    """layers: list of dicts with tensors wqkv, wo, wgu, wd, g_attn, g_ffn. Returns (handle, keepalive)."""
    arr = (LayerWeightsC * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = LayerWeightsC(*[L[k].data_ptr() for k in ("wqkv", "wo", "wgu", "wd", "g_attn", "g_ffn")])
    w = WeightsC(embed.data_ptr(), head.data_ptr(), g_final.data_ptr(), arr)
    out = C.c_void_p()
    _check(load_library().specs_model_create(ctx, C.byref(desc), C.byref(w), C.byref(out)), "specs_model_create")
    return out


def specs_model_destroy(m):
    _check(load_library().specs_model_destroy(m), "specs_model_destroy")


def specs_prefix_create(ctx, model, lens_host, lens_dev, page_tokens, kv_pool, num_pages, page_table, h_last):
    import torch
    B = len(lens_host)
    lens_arr = (C.c_int32 * B)(*[int(x) for x in lens_host])
    out = C.c_void_p()
    _check(load_library().specs_prefix_create(ctx, model, B, lens_arr, _ptr(lens_dev, torch.int32), page_tokens,
                                              _ptr(kv_pool), num_pages, _ptr(page_table, torch.int32),
                                              page_table.shape[1], _ptr(h_last, torch.float32), C.byref(out)),
           "specs_prefix_create")
    return out


def specs_prefix_destroy(p):
    _check(load_library().specs_prefix_destroy(p), "specs_prefix_destroy")


def specs_prefill(ctx, model, prefix, prefix_tokens):
    import torch
    _check(load_library().specs_prefill(ctx, model, prefix, _ptr(prefix_tokens, torch.int32)), "specs_prefill")


def specs_score_blocks(ctx, model, prefix, cand, out, tok_logp=None):
    import torch
    B, n, L = cand.shape
    _check(load_library().specs_score_blocks(ctx, model, prefix, _ptr(cand, torch.int32), n, L,
                                             _ptr(out, torch.float32), _ptr(tok_logp, torch.float32, True)),
           "specs_score_blocks")


def specs_score_target_and_reward(ctx_target, target, p_target, ctx_prm, prm, p_prm, cand, logp_target, reward,
                                  tok_logp_target=None):
    import torch
    B, n, L = cand.shape
    _check(load_library().specs_score_target_and_reward(
        ctx_target, target, p_target, ctx_prm, prm, p_prm, _ptr(cand, torch.int32), n, L,
        _ptr(logp_target, torch.float32), _ptr(tok_logp_target, torch.float32, True), _ptr(reward, torch.float32)),
        "specs_score_target_and_reward")


def specs_score_blocks_static(ctx, model, prefix, cand, out, tok_logp=None):
    import torch
    B, n, L = cand.shape
    _check(load_library().specs_score_blocks_static(ctx, model, prefix, _ptr(cand, torch.int32), n, L,
                                                    _ptr(out, torch.float32), _ptr(tok_logp, torch.float32, True)),
           "specs_score_blocks_static")


def specs_generate_blocks(ctx, model, prefix, u, cand, logp, tok_logp=None, vocab_limit=0):
    """u [B, n, L] float64 uniforms; cand [B, n, L] int32 (out), logp [B, n] (out), tok_logp [B, n, L] (out) or None."""
    import torch
    B, n, L = cand.shape
    assert tuple(u.shape) == (B, n, L) and tuple(logp.shape) == (B, n)
    _check(load_library().specs_generate_blocks(ctx, model, prefix, n, L, int(vocab_limit), _ptr(u, torch.float64),
                                                _ptr(cand, torch.int32), _ptr(logp, torch.float32),
                                                _ptr(tok_logp, torch.float32, True)), "specs_generate_blocks")


def specs_commit_block(ctx, model, prefix, chosen_host):
    arr = (C.c_int32 * len(chosen_host))(*[int(x) for x in chosen_host])
    _check(load_library().specs_commit_block(ctx, model, prefix, arr), "specs_commit_block")


def specs_commit_block_dev(ctx, model, prefix, chosen_dev):
    import torch
    _check(load_library().specs_commit_block_dev(ctx, model, prefix, _ptr(chosen_dev, torch.int32)),
           "specs_commit_block_dev")


def specs_select_and_switch(ctx, logp_target, logp_draft, reward, beta, tau, u, gen_is_draft, idx, mask=None,
                            max_reward=None):
    import torch
    B, n = logp_target.shape
    _check(load_library().specs_select_and_switch(ctx, _ptr(logp_target, torch.float32), _ptr(logp_draft, torch.float32),
                                                  _ptr(reward, torch.float32), _ptr(mask, torch.uint8, True), B, n,
                                                  float(beta), float(tau), _ptr(u, torch.float64),
                                                  _ptr(gen_is_draft, torch.uint8), _ptr(idx, torch.int32),
                                                  _ptr(max_reward, torch.float32, True)), "specs_select_and_switch")


def specs_path_counts(reset=False):
    """{path class: launches} of this process since the counters were last reset."""
    arr = (C.c_int32 * len(PATH_CLASSES))()
    _check(load_library().specs_path_counts(arr, 1 if reset else 0), "specs_path_counts")
    return {k: arr[i] for i, k in enumerate(PATH_CLASSES)}


def specs_subsample(ctx, logp_target, logp_gen, reward, betas, u, idx, mask=None, max_reward=None):
    import torch
    B, n = logp_target.shape
    nb = len(betas)
    barr = (C.c_float * nb)(*[float(b) for b in betas])
    _check(load_library().specs_subsample(ctx, _ptr(logp_target, torch.float32), _ptr(logp_gen, torch.float32),
                                          _ptr(reward, torch.float32), _ptr(mask, torch.uint8, True), B, n, barr, nb,
                                          _ptr(u, torch.float64), _ptr(idx, torch.int32),
                                          _ptr(max_reward, torch.float32, True)), "specs_subsample")


def _dt(t):
    import torch
    return SPECS_BF16 if t.dtype == torch.bfloat16 else SPECS_F32


def specs_op_linear(ctx, A, Wt, C_out, accumulate=False):
    import torch
    M, K = A.shape
    N = Wt.shape[0]
    assert Wt.shape[1] == K and C_out.shape == (M, N) and A.dtype == Wt.dtype
    _check(load_library().specs_op_linear(ctx, _dt(A), _ptr(A), _ptr(Wt), M, N, K, _ptr(C_out, torch.float32),
                                          1 if accumulate else 0), "specs_op_linear")


def specs_op_gate_up(ctx, A, Wgu, act):
    M, K = A.shape
    F = Wgu.shape[0] // 2
    assert Wgu.shape[1] == K and act.shape == (M, F) and A.dtype == Wgu.dtype == act.dtype
    _check(load_library().specs_op_gate_up(ctx, _dt(A), _ptr(A), _ptr(Wgu), M, F, K, _ptr(act)), "specs_op_gate_up")


def specs_op_lmhead_logprob(ctx, A, Wt, tok, tok_logp):
    import torch
    M, K = A.shape
    V = Wt.shape[0]
    assert Wt.shape[1] == K and tok.shape == (M,) and tok_logp.shape == (M,) and A.dtype == Wt.dtype
    _check(load_library().specs_op_lmhead_logprob(ctx, _dt(A), _ptr(A), _ptr(Wt), _ptr(tok, torch.int32), M, V, K,
                                                  _ptr(tok_logp, torch.float32)), "specs_op_lmhead_logprob")


def specs_op_attention(ctx, model, prefix, layer, q, kb, vb, n, L, out):
    _check(load_library().specs_op_attention(ctx, model, prefix, layer, _ptr(q), _ptr(kb), _ptr(vb), n, L, _ptr(out)),
           "specs_op_attention")


def specs_op_qkv_rope(ctx, model, prefix, A, Wqkv, n, L, q, kblk, vT):
    _check(load_library().specs_op_qkv_rope(ctx, model, prefix, _ptr(A), _ptr(Wqkv), n, L, _ptr(q), _ptr(kblk), _ptr(vT)),
           "specs_op_qkv_rope")


def specs_strerror(code):
    return load_library().specs_strerror(code).decode()
