"""Counter-based generator: value(seed, stream-name, index) with no sequential state.

Every draw is a pure function of (seed, name, counter), so any slice of any tensor can be
produced on its own (the CPU oracle asks for single embedding rows of a 7B model) and the
numpy implementation here and the torch implementation (used to fill device memory without
a PCIe copy of tens of GB) give bit-identical results: the only floating-point step is a
table lookup.

Integer mixing: two rounds of the 32-bit "lowbias32" finaliser (C. Wellons, hash-prospector,
public domain) keyed by two words derived from (seed, name) with BLAKE2b.
Normal draws: inverse-CDF table with 2**20 equiprobable cells, cell k holding
Phi^{-1}((k + 1/2) / 2**20), scaled by std and (for bf16 tensors) rounded once to bf16 by
round-to-nearest-even; a draw is table[hash >> 12].
"""
import hashlib
import numpy as np

_M32 = 0xFFFFFFFF
_TABLE_BITS = 20


def stream_key(seed: int, name: str):
    h = hashlib.blake2b(f"{seed}:{name}".encode(), digest_size=8).digest()
    return int.from_bytes(h[:4], "little"), int.from_bytes(h[4:], "little")


def _lowbias32_np(x):
    # uint32 arrays: numpy multiplication wraps modulo 2**32
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return x


def _hash_counters(seed, name, ctr_u32):
    k1, k2 = stream_key(seed, name)
    x = ctr_u32 ^ np.uint32(k1)
    x = _lowbias32_np(x)
    x += np.uint32(k2)
    return _lowbias32_np(x)


def raw_u32(seed: int, name: str, start: int, count: int) -> np.ndarray:
    """uint32 draws for counters start .. start+count-1 (counters taken modulo 2**32)."""
    ctr = (np.arange(start, start + count, dtype=np.uint64) & np.uint64(_M32)).astype(np.uint32)
    return _hash_counters(seed, name, ctr)


def raw_u32_at(seed: int, name: str, idx: np.ndarray) -> np.ndarray:
    return _hash_counters(seed, name, (idx.astype(np.uint64) & np.uint64(_M32)).astype(np.uint32))


def bf16_round_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result still stored as float32."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000))
    return r.view(np.float32)


_table_cache = {}


def normal_table(std: float, dtype: str) -> np.ndarray:
    """float32 table of 2**20 normal quantiles times std; bf16-valued when dtype == 'bf16'."""
    key = (float(std), dtype)
    if key not in _table_cache:
        from scipy.special import ndtri
        n = 1 << _TABLE_BITS
        z = ndtri((np.arange(n, dtype=np.float64) + 0.5) / n)
        t = (z * std).astype(np.float32)
        if dtype == "bf16":
            t = bf16_round_f32(t)
        elif dtype != "f32":
            raise ValueError(dtype)
        _table_cache[key] = t
    return _table_cache[key]


def normal_tensor(seed, name, shape, std, dtype, rows=None, device=None):
    """N(0, std) tensor named `name`, row-major counters.

    numpy float32 array (bf16-valued for dtype 'bf16') when device is None; otherwise a torch
    tensor (bfloat16 / float32) created on `device` with identical values.
    rows: optional 1-D integer array selecting rows of a 2-D tensor (numpy path only).
    """
    shape = tuple(int(s) for s in shape)
    table = normal_table(std, dtype)
    if device is None:
        if rows is not None:
            ncol = shape[1]
            idx = (np.asarray(rows, dtype=np.uint64)[:, None] * np.uint64(ncol)
                   + np.arange(ncol, dtype=np.uint64)[None, :])
            h = raw_u32_at(seed, name, idx.reshape(-1))
            return table[h >> np.uint32(32 - _TABLE_BITS)].reshape(len(rows), ncol)
        total = int(np.prod(shape))
        out = np.empty(total, dtype=np.float32)
        step = 1 << 22

        def fill(s0):
            c = min(step, total - s0)
            out[s0:s0 + c] = table[raw_u32(seed, name, s0, c) >> np.uint32(32 - _TABLE_BITS)]

        starts = range(0, total, step)
        if total > step:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=8) as ex:
                list(ex.map(fill, starts))
        else:
            for s0 in starts:
                fill(s0)
        return out.reshape(shape)
    import torch
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ttab = _torch_table(std, dtype, device)
    k1, k2 = stream_key(seed, name)
    total = int(np.prod(shape))
    out = torch.empty(total, dtype=tdt, device=device)
    step = 1 << 26
    for s in range(0, total, step):
        c = min(step, total - s)
        x = torch.arange(s, s + c, dtype=torch.int64, device=device)
        x = (x & _M32) ^ k1
        x = _lowbias32_t(x)
        x = (x + k2) & _M32
        x = _lowbias32_t(x)
        out[s:s + c] = ttab[x >> (32 - _TABLE_BITS)]
    return out.reshape(shape)


_ttab_cache = {}


def _torch_table(std, dtype, device):
    import torch
    key = (float(std), dtype, str(device))
    if key not in _ttab_cache:
        t = torch.from_numpy(normal_table(std, dtype).copy()).to(device)
        if dtype == "bf16":
            t = t.to(torch.bfloat16)          # exact: values are already bf16-representable
        _ttab_cache[key] = t
    return _ttab_cache[key]


def _lowbias32_t(x):
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32           # int64 product may wrap; the low 32 bits are exact
    x = x ^ (x >> 16)
    return x


def uniform_f64(seed, name, count, start=0) -> np.ndarray:
    """float64 uniforms in [0, 1) with 53 random bits each (two 32-bit draws per value)."""
    h = raw_u32(seed, name, 2 * start, 2 * count)
    hi = h[0::2] >> np.uint32(5)      # 27 bits
    lo = h[1::2] >> np.uint32(6)      # 26 bits
    return (hi.astype(np.float64) * 67108864.0 + lo.astype(np.float64)) / 9007199254740992.0


def uniform_tokens(seed, name, count, vocab) -> np.ndarray:
    h = raw_u32(seed, name, 0, count)
    return ((h.astype(np.uint64) * np.uint64(vocab)) >> np.uint64(32)).astype(np.int32)


_zipf_cache = {}


def zipf_tokens(seed, name, count, vocab, s=1.1) -> np.ndarray:
    """ids with p(id = k-1) proportional to k**-s, k = 1..vocab; inverse CDF on a float64 table."""
    key = (int(vocab), float(s))
    if key not in _zipf_cache:
        w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
        cdf = np.cumsum(w)
        _zipf_cache[key] = cdf / cdf[-1]
    cdf = _zipf_cache[key]
    u = (raw_u32(seed, name, 0, count).astype(np.float64) + 0.5) / 4294967296.0
    return np.minimum(np.searchsorted(cdf, u, side="left"), vocab - 1).astype(np.int32)


def permutation(seed, name, n) -> np.ndarray:
    """A permutation of 0..n-1: stable argsort of n hashed keys."""
    return np.argsort(raw_u32(seed, name, 0, n), kind="stable").astype(np.int32)
