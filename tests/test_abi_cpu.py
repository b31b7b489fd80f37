"""CPU-side checks of the boundary: the built library exports every symbol the
header declares, the binding lists the same names, and without a GPU the entry
points fail loudly instead of falling back to anything."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2511_21759_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def libpath():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_21759_amd.build import build_library
        build_library()
    return binding.LIB_PATH


def header_symbols():
    text = open(os.path.join(ROOT, "include", "odb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(odb_[a-z_]+)\s*\(", text)))


def test_header_declares_the_two_calls_of_the_path():
    syms = header_symbols()
    assert "odb_prefill" in syms and "odb_block_step" in syms
    assert sorted(binding.SYMBOLS) == syms


def test_library_exports_every_declared_symbol(libpath):
    lib = ctypes.CDLL(libpath)
    for s in header_symbols():
        assert hasattr(lib, s), s


def test_no_torch_types_in_the_abi():
    text = open(os.path.join(ROOT, "include", "odb.h")).read()
    assert "torch" not in re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert "at::" not in text and "#include <hip" not in text


def test_strerror_and_argument_validation_without_gpu(libpath):
    lib = binding.lib()
    assert lib.odb_strerror(0) == b"ok"
    assert lib.odb_strerror(-1) == b"invalid argument"
    out = ctypes.c_void_p()
    # NULL config is rejected before anything touches the device
    assert lib.odb_model_create(None, None, ctypes.byref(out)) == -1
    assert b"NULL" in lib.odb_last_error()
    bad = dict(workloads.MODEL_SHAPES["tiny"], head_dim=48)
    with pytest.raises(binding.OdbError):
        binding.odb_model_create(bad)
    assert lib.odb_prefill(None, None, None, 1, 0, None, None, None) == -1
    assert lib.odb_block_step(None, None, None, 0, 1, 1, 0.5, None, None, None, None) == -1


def test_product_path_fails_loudly_without_a_gpu(libpath):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(binding.OdbError):
        binding.odb_model_create(workloads.MODEL_SHAPES["tiny"])


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_21759_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no oracle", "").replace("CPU oracle", "") or f == "workloads.py", f


def test_workloads_are_seeded_and_shaped():
    a, b = workloads.config1(), workloads.config2()
    assert a.tokens.shape == (1, 512) and a.drafts.shape == (1, 1, 32) and a.block_off == 256
    assert b.drafts.shape == (1, 4, 32) and np.array_equal(a.tokens, b.tokens)
    assert np.array_equal(b.drafts[0, 0], b.tokens[0, 256:288])
    m = workloads.MODEL_SHAPES["8b"]["mask_id"]
    for s, extra in zip(range(1, 4), (1, 1, 2)):
        assert ((b.drafts[0, 0] == m).sum() - (b.drafts[0, s] == m).sum()) == extra
    assert np.array_equal(workloads.config1().drafts, a.drafts)
    c0 = workloads.config0()
    assert c0.tokens.shape == (1, 192) and (c0.tokens[0, 128:] == 1023).all() and c0.drafts.shape == (1, 1, 16)
    c4 = workloads.config4()
    assert c4.tokens.shape == (4, 3072) and c4.drafts.shape == (4, 8, 64) and c4.block_off == 2048
    assert workloads.config3(256).shape == (1, 768)


def test_bench_reads_the_gate_up_row_of_every_tracked_profile():
    """bench.py quotes the kernel-trace average and the measured HBM bytes of the gate/up GEMM from the tracked
    rocprofv3 summaries: every one of them must hold a row that its parser finds, with figures of a plausible size."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("odb_bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for name, (lo_us, hi_us) in {"config1": (20, 60), "config2": (30, 80), "config3": (100, 300), "config4": (200, 600)}.items():
        avg_us, traffic, rel = bench.profile_figures(name)
        assert avg_us is not None and lo_us < avg_us < hi_us, (name, avg_us, rel)
        assert traffic is not None and 1.9e8 < traffic < 2e9, (name, traffic, rel)
