"""The seeded input generators: determinism, numpy/torch bit-equality, distribution sanity."""
import numpy as np
import torch
import workload as W
from workload.configs import HostWeights, device_tensor


def test_numpy_and_torch_generators_agree_bit_for_bit():
    c = W.get_config("c2_small")
    hw = HostWeights(c.target)
    lay = hw.layer(3)
    t = device_tensor(c.target, 0, "L3/wd", lay["wd"].shape, "cpu")
    assert t.dtype == torch.bfloat16 and np.array_equal(t.float().numpy(), lay["wd"])
    c1 = W.get_config("c1_tiny")
    t = device_tensor(c1.target, 0, "embed", (512, 64), "cpu")
    assert t.dtype == torch.float32 and np.array_equal(t.numpy(), HostWeights(c1.target).embed_rows(np.arange(512)))
    rows = hw.embed_rows([5, 32767, 0])
    assert np.array_equal(rows[1], device_tensor(c.target, 0, "embed", (32768, 1024), "cpu")[32767].float().numpy())


def test_weight_statistics_and_stream_independence():
    c = W.get_config("c2_small")
    a, b = HostWeights(c.target).layer(0)["wg"], HostWeights(c.prm).layer(0)["wg"]
    assert abs(a.std() - 0.02) < 2e-4 and abs(a.mean()) < 1e-4
    assert abs(np.corrcoef(a.ravel()[:100000], b.ravel()[:100000])[0, 1]) < 0.02
    assert np.array_equal(W.bf16_round_f32(a), a)            # bf16-valued


def test_tokens_lengths_pages_uniforms():
    c5 = W.get_config("c5_7b_batched")
    lens = c5.prefix_lens()
    assert lens.shape == (32,) and lens.min() >= 1024 and lens.max() < 8192
    table, total = c5.page_table()
    used = table[table >= 0]
    assert len(used) == total == len(set(used.tolist())) and used.max() == total - 1
    assert np.all((table >= 0).sum(1) == (lens + 15) // 16)
    cand = c5.candidates()
    assert cand.shape == (32, 8, 64) and cand.min() >= 0 and cand.max() < 151936
    assert (cand == 0).mean() > 0.05                          # Zipf(1.1): rank 1 carries ~9% of the mass
    u = c5.uniforms()
    assert u.shape == (32, 4) and u.min() >= 0 and u.max() < 1
    assert np.array_equal(u, c5.uniforms())
    c1 = W.get_config("c1_tiny")
    assert c1.candidates().shape == (1, 4, 16) and c1.candidates().max() < 512
    assert [len(t) for t in W.get_config("c4_7b").prefix_tokens()] == [4096]
