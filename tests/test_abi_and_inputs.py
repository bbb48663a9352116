"""CPU-side checks: the C-ABI library loads and exports every symbol the header
declares, argument errors that need no GPU, and the seeded input generators."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2509_05576_amd as fobq
    if not os.path.exists(fobq.lib_path()):
        from paper_2509_05576_amd import build
        build.build(verbose=False)
    return fobq, fobq.load_library()


def test_library_exports_every_declared_symbol():
    _, lib = _lib()
    header = open(os.path.join(ROOT, "include", "fobq.h")).read()
    names = sorted(set(re.findall(r"^(?:int|const char\*)\s+(fobq_[a-z_0-9]+)\s*\(", header, flags=re.M)))
    assert {"fobq_create", "fobq_destroy", "fobq_last_error", "fobq_hessian_begin", "fobq_hessian_accumulate",
            "fobq_hessian_accumulate_conv", "fobq_hessian_finalize", "fobq_quantize_layer",
            "fobq_quantize_layer_enqueue", "fobq_finish", "fobq_spd_inverse", "fobq_sensitivity",
            "fobq_profile_enable", "fobq_profile_get", "fobq_profile_reset"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"libfobq.so does not export {n}"


def test_null_context_is_rejected_without_touching_a_gpu():
    fobq, lib = _lib()
    null = ctypes.c_void_p(None)
    assert lib.fobq_hessian_begin(null, 8) == fobq.EINVAL
    assert lib.fobq_hessian_accumulate(null, null, 1, 1) == fobq.EINVAL
    assert lib.fobq_hessian_accumulate_conv(null, null, 1, 1, 1, 1, 1, 1, 0) == fobq.EINVAL
    assert lib.fobq_hessian_finalize(null, null) == fobq.EINVAL
    assert lib.fobq_quantize_layer(null, null, 1, 1, null, None, None) == fobq.EINVAL
    assert lib.fobq_quantize_layer_enqueue(null, null, 1, 1, null, None, None) == fobq.EINVAL
    assert lib.fobq_finish(null) == fobq.EINVAL
    assert lib.fobq_spd_inverse(null, null, 1, null) == fobq.EINVAL
    assert lib.fobq_profile_enable(null, 1) == fobq.EINVAL
    assert lib.fobq_destroy(null) == fobq.OK
    assert lib.fobq_last_error(null) == b"context is NULL"
    assert lib.fobq_create(None, 0, null) == fobq.EINVAL


def test_binding_rejects_host_tensors():
    torch = pytest.importorskip("torch")
    fobq, _ = _lib()
    with pytest.raises(TypeError):
        fobq.fobq_hessian_accumulate(1, torch.zeros(4, 4))
    with pytest.raises(TypeError):
        fobq.fobq_quantize_layer(1, torch.zeros(4, 4))


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_05576_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"


# ---------------------------------------------------------------- generators
def test_generator_is_counter_based_and_reproducible():
    a = workloads.normal_f64(1000, seed=3, stream=2)
    b = workloads.normal_f64(1000, seed=3, stream=2)
    assert np.array_equal(a, b)
    # any slice can be produced on its own
    assert np.array_equal(workloads.normal_f64(100, 3, 2, offset=400), a[400:500])
    assert not np.array_equal(a, workloads.normal_f64(1000, seed=4, stream=2))
    assert not np.array_equal(a, workloads.normal_f64(1000, seed=3, stream=3))


def test_generator_moments():
    z = workloads.normal_f64(400000, seed=0, stream=9)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs(np.mean(z ** 3)) < 0.03 and abs(np.mean(z ** 4) - 3.0) < 0.1
    r = workloads.relu_normal_f32((1000, 100), 0, 9)
    assert r.dtype == np.float32 and r.min() == 0.0 and abs(r.mean() - 0.3989) < 0.01


def test_im2col_matches_a_direct_loop():
    rng = np.random.default_rng(0)
    maps = rng.standard_normal((2, 5, 4, 3)).astype(np.float32)
    for k, stride, pad in [(3, 1, 1), (1, 1, 0), (3, 2, 1)]:
        X = workloads.im2col(maps, k, stride, pad)
        ho = (5 + 2 * pad - k) // stride + 1
        wo = (4 + 2 * pad - k) // stride + 1
        assert X.shape == (3 * k * k, 2 * ho * wo)
        for c in range(3):
            for ky in range(k):
                for kx in range(k):
                    for n in range(2):
                        for y in range(ho):
                            for x in range(wo):
                                yy, xx = y * stride + ky - pad, x * stride + kx - pad
                                v = maps[n, yy, xx, c] if 0 <= yy < 5 and 0 <= xx < 4 else 0.0
                                assert X[c * k * k + ky * k + kx, n * ho * wo + y * wo + x] == v


def test_config_shapes_and_model_totals():
    c = workloads.configs()
    assert (c["c1_tiny"].d_row, c["c1_tiny"].d_col, c["c1_tiny"].n) == (64, 128, 512)
    s = c["c2_resnet50_3x3"]
    assert (s.d_row, s.d_col, s.n, s.bits) == (256, 2304, 25088, 4)
    assert (c["c5_large_d"].d_col, c["c5_large_d"].group, c["c5_large_d"].bits) == (4608, 128, 3)
    W = c["c1_tiny"].make_w()
    X = c["c1_tiny"].make_x()
    assert W.shape == (64, 128) and X.shape == (128, 512) and W.dtype == np.float32
    assert abs(W.std() - 0.05) < 0.002 and X.min() == 0.0
    r50 = workloads.sweep_layers("resnet50")
    y5 = workloads.sweep_layers("yolov5s")
    assert len(r50) == 54 and len(y5) == 60
    assert abs(sum(l.weights for l in r50) / 1e6 - 25.50) < 0.05
    assert abs(sum(l.weights for l in y5) / 1e6 - 7.22) < 0.05


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before it touches the GPU."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""
