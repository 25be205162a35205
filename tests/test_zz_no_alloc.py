"""specs_score_blocks_static (working buffers in the library's static device scratch, no workspace, no allocation)
against specs_score_blocks on the same inputs, through the raw C ABI: two calls in a row, the second smaller."""
import ctypes as C

import numpy as np
import pytest
import torch

import workload as W

pytestmark = pytest.mark.gpu


def _score(lib, fn, dm, pre, cand, with_tokens):
    Bn, n, L = cand.shape
    out = torch.full((Bn, n), float("nan"), dtype=torch.float32, device=cand.device)
    tok = torch.full((Bn, n, L), float("nan"), dtype=torch.float32, device=cand.device) if with_tokens else None
    rc = getattr(lib, fn)(dm.ctx, dm.model, pre.handle, C.c_void_p(cand.data_ptr()), n, L, C.c_void_p(out.data_ptr()),
                          C.c_void_p(tok.data_ptr()) if with_tokens else None)
    assert rc == 0, (fn, rc)
    torch.cuda.synchronize()
    st = C.c_int(-1)
    assert lib.specs_ctx_status(dm.ctx, C.byref(st)) == 0 and st.value == 0
    return out.cpu().numpy(), (tok.cpu().numpy() if with_tokens else None)


@pytest.mark.parametrize("name", ["c1_tiny", "c2_small"])
def test_static_scratch_entry_point_equals_the_workspace_one(name):
    from paper_2506_15733_amd import binding, synthetic
    lib = binding.load_library()
    wl = W.get_config(name)
    step = synthetic.ScoringStep(wl, concurrent=False)
    step.prefill()
    torch.cuda.synchronize()
    small = torch.from_numpy(np.ascontiguousarray(wl.candidates()[:, :3, :wl.L - 5])).to(step.device)
    try:
        for cand in (step.cand, small):                      # the second call is smaller than the first
            for role in step.ROLES:
                dm, pre = step.models[role], step.prefixes[role]
                lm = dm.desc.head == "lm"
                want = _score(lib, "specs_score_blocks", dm, pre, cand, lm)
                got = _score(lib, "specs_score_blocks_static", dm, pre, cand, lm)
                assert np.isfinite(want[0]).all()
                assert np.array_equal(got[0], want[0]), (name, role, tuple(cand.shape))
                if lm:
                    assert np.array_equal(got[1], want[1]), (name, role, tuple(cand.shape))
        # the block scored in the static scratch cannot be committed, and the workspace entry point still can be
        dm, pre = step.models["target"], step.prefixes["target"]
        chosen = (C.c_int32 * wl.B)(*([0] * wl.B))
        assert lib.specs_commit_block(dm.ctx, dm.model, pre.handle, chosen) == 1      # SPECS_EINVAL
    finally:
        step.close()


def test_static_scratch_rejects_what_does_not_fit():
    """A 1.5B-shaped pass needs more than the static scratch holds: SPECS_EWORKSPACE, nothing launched."""
    from paper_2506_15733_amd import binding, synthetic
    lib = binding.load_library()
    wl = W.get_config("c3_1p5b")
    desc = W.configs.scaled(wl, target=W.ModelDesc("target", 1, 1536, 12, 2, 128, 8960, 151936)).target
    stream = torch.cuda.current_stream()
    dm = synthetic.DeviceModel(desc, "cuda:0", stream, wl.n * wl.L, wl.n)
    table, pages = wl.page_table()
    pre = synthetic.DevicePrefix(dm, wl.prefix_lens(), table, pages, wl.page_tokens)
    cand = torch.from_numpy(wl.candidates()).to("cuda:0")
    out = torch.zeros((1, wl.n), dtype=torch.float32, device="cuda:0")
    need = binding.specs_workspace_bytes(dm.cdesc, wl.n * wl.L, wl.n)
    assert need > (32 << 20)
    rc = lib.specs_score_blocks_static(dm.ctx, dm.model, pre.handle, C.c_void_p(cand.data_ptr()), wl.n, wl.L,
                                       C.c_void_p(out.data_ptr()), None)
    assert rc == 7                                           # SPECS_EWORKSPACE
    torch.cuda.synchronize()
    pre.close()
    dm.close()
