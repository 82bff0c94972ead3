"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.
Integers (sorted keys, stable order, unique rows, segment starts, the set of updated rows) must agree
bit for bit; floats within the tolerance stated in gpu_harness."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def test_c1_exact_config(H):
    # 1 table, 100000 x 64 fp32, B=512, L=20, uniform ids, sum pooling, lr=0.01, eps=1e-8, seed 0; c in {1, 4}
    for c in (1.0, 4.0):
        cfg = W.config("C1", c=c)
        reps = H.run_config(cfg, steps=2)
        print("C1 c=%g" % c, reps, flush=True)
        assert reps[0]["U"] > 9000


def test_c2_full_size(H):
    cfg = W.config("C2")
    reps = H.run_config(cfg, steps=2)
    print("C2", reps, flush=True)
    assert reps[0]["max_seg"] > 1000          # the Zipf head makes long segments that take the split path


@pytest.mark.parametrize("name,kw", [
    ("C3", dict(T=12, B=512, rows_scale=2e-3)),       # mixed D in {64,128,256}, hot rows
    ("C4", dict(T=8, B=256, rows_scale=1e-3)),        # fp16 tables, D in {128,256}
    ("C5", dict(T=32, B=1024, rows_scale=1e-3)),      # mean pooling, D=128 and D=32, long-tailed bag lengths
    ("C5I", dict(T=32, B=1024, rows_scale=1e-3)),     # the same tables, the big ones spread among the small ones
])
def test_scaled_configs(H, name, kw):
    cfg = W.config(name, c=2.0, **kw)
    reps = H.run_config(cfg, steps=2, state_kind="hash")
    print(name, reps, flush=True)


def test_fp16_and_mean_variants_of_c2_shape(H):
    for wd, pool in (("f16", "sum"), ("f32", "mean"), ("f16", "mean")):
        cfg = W.config("C2", T=6, B=512, rows_scale=0.05, weight_dtype=wd, pooling=pool, c=4.0)
        reps = H.run_config(cfg, steps=1, state_kind="hash")
        print(wd, pool, reps, flush=True)
