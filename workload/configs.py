"""Shape presets of the five benchmark configurations and the seeded inputs that go with them.

Nothing here computes anything of the method; it only names shapes and draws inputs.
Weights: N(0, 0.02) for every matrix, RMSNorm gains = 1, no biases, lm_head untied from the
embedding; one generator stream per tensor, named "<role>/<tensor>" or "<role>/L<l>/<tensor>".
All matrices are stored [out_features, in_features] row-major (y = x W^T).
"""
from dataclasses import dataclass, field, replace
from typing import Tuple
import numpy as np
from . import rng

WEIGHT_STD = 0.02


@dataclass(frozen=True)
class ModelDesc:
    role: str                 # generator stream prefix: "target" | "draft" | "prm"
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str = "bf16"       # operand type: "bf16" | "f32"
    head: str = "lm"          # "lm" (vocab projection) | "prm" (scalar head)
    rope_base: float = 10000.0
    rms_eps: float = 1e-6

    @property
    def qkv_rows(self):
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def kv_bytes_per_token(self):
        return 2 * self.n_layers * self.n_kv_heads * self.head_dim * (2 if self.dtype == "bf16" else 4)


def weight_shapes(m: ModelDesc):
    """name -> shape of every tensor of a model (per-layer names carry an 'L{l}/' prefix)."""
    per_layer = {
        "wqkv": (m.qkv_rows, m.d_model),                    # rows: Hq q-heads, Hkv k-heads, Hkv v-heads
        "wo": (m.d_model, m.n_q_heads * m.head_dim),
        "wg": (m.ffn, m.d_model),
        "wu": (m.ffn, m.d_model),
        "wd": (m.d_model, m.ffn),
    }
    top = {"embed": (m.vocab, m.d_model)}
    top["head"] = (m.vocab, m.d_model) if m.head == "lm" else (1, m.d_model)
    return top, per_layer


class HostWeights:
    """Lazily generated numpy weights of one model (float32 arrays, bf16-valued for bf16 models)."""

    def __init__(self, desc: ModelDesc, seed: int = 0):
        self.desc, self.seed = desc, seed
        self._top, self._per_layer = weight_shapes(desc)

    def _gen(self, name, shape, rows=None):
        return rng.normal_tensor(self.seed, f"{self.desc.role}/{name}", shape, WEIGHT_STD,
                                 self.desc.dtype, rows=rows)

    def embed_rows(self, ids):
        return self._gen("embed", self._top["embed"], rows=np.asarray(ids).reshape(-1))

    def head(self):
        return self._gen("head", self._top["head"])

    def layer(self, l):
        return {k: self._gen(f"L{l}/{k}", s) for k, s in self._per_layer.items()}

    def gains(self):
        d = self.desc.d_model
        return {"attn": np.ones(d), "ffn": np.ones(d), "final": np.ones(d)}


def device_tensor(desc: ModelDesc, seed: int, name: str, shape, device):
    """The same tensor as HostWeights would give, created directly in device memory (torch)."""
    return rng.normal_tensor(seed, f"{desc.role}/{name}", shape, WEIGHT_STD, desc.dtype, device=device)


@dataclass(frozen=True)
class Workload:
    name: str
    target: ModelDesc
    draft: ModelDesc
    prm: ModelDesc
    B: int
    n: int
    L: int
    prefix_len: int                   # fixed P, or 0 when lengths are drawn (lens_range)
    betas: Tuple[float, ...]
    token_dist: str                   # "uniform" | "zipf"
    lens_range: Tuple[int, int] = (0, 0)
    page_tokens: int = 16
    seed: int = 0
    u_seed: int = 1

    @property
    def token_vocab(self):
        return min(self.target.vocab, self.draft.vocab, self.prm.vocab)

    def models(self):
        return {"target": self.target, "draft": self.draft, "prm": self.prm}

    def prefix_lens(self) -> np.ndarray:
        if self.prefix_len:
            return np.full(self.B, self.prefix_len, dtype=np.int32)
        lo, hi = self.lens_range
        u = rng.uniform_f64(self.seed, "lens", self.B)
        return np.floor(lo * (hi / lo) ** u).astype(np.int32)

    def _tokens(self, stream, count):
        if self.token_dist == "uniform":
            return rng.uniform_tokens(self.seed, stream, count, self.token_vocab)
        return rng.zipf_tokens(self.seed, stream, count, self.token_vocab, 1.1)

    def prefix_tokens(self):
        """list of B int32 arrays (ragged)."""
        lens = self.prefix_lens()
        flat = self._tokens("tokens/prefix", int(lens.sum()))
        offs = np.concatenate([[0], np.cumsum(lens)])
        return [flat[offs[b]:offs[b + 1]] for b in range(self.B)]

    def candidates(self) -> np.ndarray:
        return self._tokens("tokens/cand", self.B * self.n * self.L).reshape(self.B, self.n, self.L)

    def page_table(self, extra_tokens: int = 0):
        """(table [B, max_pages] int32 padded with -1, num_pages): shuffled physical page order."""
        lens = self.prefix_lens() + extra_tokens
        need = (lens + self.page_tokens - 1) // self.page_tokens
        total = int(need.sum())
        perm = rng.permutation(self.seed, "pages", total)
        table = np.full((self.B, int(need.max())), -1, dtype=np.int32)
        o = 0
        for b in range(self.B):
            table[b, :need[b]] = perm[o:o + need[b]]
            o += need[b]
        return table, total

    def uniforms(self) -> np.ndarray:
        """float64 [B, len(betas)], row-major from the u_seed stream."""
        return rng.uniform_f64(self.u_seed, "subsample/u", self.B * len(self.betas)).reshape(self.B, -1)

    def synthetic_scores(self, B=None, n=None):
        """Directly synthesised score vectors that make beta matter: lt - ld ~ N(0, 5^2), r ~ U(0,1)."""
        B = B or self.B
        n = n or self.n
        z = rng.normal_table(1.0, "f32")[rng.raw_u32(self.seed, "synth/ratio", 0, B * n) >> np.uint32(12)]
        ld = -50.0 + 3.0 * rng.normal_table(1.0, "f32")[rng.raw_u32(self.seed, "synth/ld", 0, B * n) >> np.uint32(12)]
        lt = (ld + 5.0 * z).astype(np.float32)
        r = rng.uniform_f64(self.seed, "synth/r", B * n).astype(np.float32)
        return lt.reshape(B, n), ld.astype(np.float32).reshape(B, n), r.reshape(B, n)


def _m(role, nl, d, hq, hkv, hd, f, v, dtype="bf16", head="lm"):
    return ModelDesc(role, nl, d, hq, hkv, hd, f, v, dtype, head)


def _trio(t, dr):
    return dict(target=_m("target", *t), draft=_m("draft", *dr), prm=_m("prm", *t, head="prm"))


_TINY = (2, 64, 4, 4, 16, 256, 512, "f32")
_TINY_D = (1, 64, 4, 4, 16, 256, 512, "f32")
_SMALL = (16, 1024, 16, 8, 64, 2816, 32768)
_SMALL_D = (4, 1024, 16, 8, 64, 2816, 32768)
_Q05 = (24, 896, 14, 2, 64, 4864, 151936)
_Q15 = (28, 1536, 12, 2, 128, 8960, 151936)
_Q7 = (28, 3584, 28, 4, 128, 18944, 152064)

CONFIGS = {
    "c1_tiny": Workload("c1_tiny", **_trio(_TINY, _TINY_D), B=1, n=4, L=16, prefix_len=32,
                        betas=(1.0,), token_dist="uniform"),
    "c2_small": Workload("c2_small", **_trio(_SMALL, _SMALL_D), B=1, n=8, L=32, prefix_len=512,
                         betas=(0.5, 1.0, 4.0), token_dist="zipf"),
    "c3_1p5b": Workload("c3_1p5b", **_trio(_Q15, _Q05), B=1, n=16, L=64, prefix_len=2048,
                        betas=(1.0,), token_dist="zipf"),
    "c4_7b": Workload("c4_7b", **_trio(_Q7, _Q15), B=1, n=16, L=128, prefix_len=4096,
                      betas=(1.0,), token_dist="zipf"),
    "c5_7b_batched": Workload("c5_7b_batched", **_trio(_Q7, _Q15), B=32, n=8, L=64, prefix_len=0,
                              lens_range=(1024, 8192), betas=(0.25, 1.0, 4.0, 16.0), token_dist="zipf"),
}


def get_config(name: str) -> Workload:
    return CONFIGS[name]


def scaled(wl: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (tests use reduced layer counts, etc.)."""
    return replace(wl, **kw)
