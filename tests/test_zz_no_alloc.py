"""odb_block_step_static: the block step for callers that cannot allocate device memory.  It runs the kernels
of odb_block_step in the library's fixed scratch area, so its outputs must equal odb_block_step's bit for bit
(the same bar as every integer output, and stricter than the floating-point one), on two calls in a row, the
second with a smaller input that finds the first call's leftovers in the area."""
import numpy as np
import pytest

from paper_2511_21759_amd import binding as B
from paper_2511_21759_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def cuda_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()


def outputs(Bn, S, b):
    return (torch.empty((Bn, S, b), dtype=torch.float32, device="cuda"),
            torch.empty((Bn, S, b), dtype=torch.int32, device="cuda"),
            torch.empty((Bn, S, b), dtype=torch.uint8, device="cuda"))


def compare(model, cache, drafts, block_off, tau, tag):
    d = cuda_i32(drafts)
    ref = [t.clone() for t in B.odb_block_step(model, cache, d, block_off, tau)]
    torch.cuda.synchronize()
    out = outputs(*drafts.shape)
    for t in out:
        t.fill_(77)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = B.odb_block_step_static(model, cache, d, block_off, tau, *out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before, "%s: the call went to the allocator" % tag
    for x, y, name in zip(got, ref, ("conf", "argmax", "unmask")):
        assert torch.equal(x, y), "%s: %s differs from odb_block_step" % (tag, name)
    assert ref[2].sum().item() >= 1
    B.odb_model_status(model)


def test_static_scratch_step_equals_block_step_on_the_tiny_model():
    shape = W.MODEL_SHAPES["tiny"]
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        B.odb_model_set_tensor(model, B.T_GF, 0, np.full(shape["d_model"], 0x4200, np.uint16))     # gain 32: tau binds
        wl = W.decode_workload(shape, 100, 92, 48, 9, 1234, batch=2)          # 2 x 9 x 48 = 864 rows, ragged key tiles
        cache = B.odb_cache_create(model, 2, wl.tokens.shape[1])
        B.odb_prefill(model, cache, cuda_i32(wl.tokens), wl.resp_off)
        compare(model, cache, wl.drafts, wl.block_off, 0.9, "tiny, 864 rows")
        # second call, smaller: fewer drafts of a shorter, ragged block (every buffer starts somewhere else in the area)
        small = np.ascontiguousarray(wl.drafts[:, :2, :20])
        compare(model, cache, small, wl.block_off, 0.9, "tiny, 80 rows after 864")
        compare(model, cache, wl.drafts[:, :1, :1].copy(), wl.block_off, 0.9, "tiny, single-token blocks")
        compare(model, cache, wl.drafts, wl.block_off, 0.5, "tiny, 864 rows again")
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)


def test_static_scratch_step_at_the_8b_width_and_its_size_limit():
    shape = dict(W.MODEL_SHAPES["8b"], n_layers=2)
    model = B.odb_model_create(shape)
    try:
        B.odb_model_init_random(model, W.WEIGHT_SEED, W.WEIGHT_STD)
        wl = W.config2()
        cache = B.odb_cache_create(model, 1, wl.tokens.shape[1])
        B.odb_prefill(model, cache, cuda_i32(wl.tokens), wl.resp_off)
        compare(model, cache, wl.drafts, wl.block_off, wl.tau, "8B width, 128 rows")
        compare(model, cache, wl.drafts[:, :1].copy(), wl.block_off, wl.tau, "8B width, 32 rows after 128")
        compare(model, cache, wl.drafts[:, :3].copy(), wl.block_off, wl.tau, "8B width, 96 rows")
        # beyond the fixed area: refused before anything is launched, outputs untouched
        big = np.ascontiguousarray(np.repeat(wl.drafts, 8, axis=1))          # 32 drafts = 1024 rows
        out = outputs(*big.shape)
        for t in out:
            t.fill_(55)
        with pytest.raises(B.OdbError, match="fixed"):
            B.odb_block_step_static(model, cache, cuda_i32(big), wl.block_off, wl.tau, *out)
        torch.cuda.synchronize()
        assert (out[0] == 55).all() and (out[1] == 55).all() and (out[2] == 55).all()
        with pytest.raises(B.OdbError):
            B.odb_block_step_static(model, cache, cuda_i32(wl.drafts), 500, wl.tau, *outputs(*wl.drafts.shape))
        B.odb_cache_destroy(cache)
    finally:
        B.odb_model_destroy(model)
