"""Host-only checks of the seeded input generator, the stored tripwire values,
and the anti-degeneracy criteria (paper, appendix "Compromised KernelBench
Tasks", filtering procedure) applied to the oracle's outputs on the small
configuration: outputs not confined to a narrow band, not constant along an
axis, and sensitive to the input seed."""
import importlib.util
import os

import numpy as np
import torch

from oracle import fdl_oracle as O
from paper_2509_14279_amd import inputs as I

HERE = os.path.dirname(os.path.abspath(__file__))


def test_configs_table():
    shapes = [(c.dtype, c.M, c.K, c.N, c.seed) for c in I.CONFIGS]
    assert shapes == [("f32", 256, 256, 256, 0), ("bf16", 8192, 1024, 4096, 1), ("f32", 3001, 771, 1537, 2),
                      ("bf16", 16384, 4096, 4096, 3), ("bf16", 65536, 2048, 8192, 4)]
    assert I.CONFIGS[3].x_mean == 50.0 and I.CONFIGS[3].x_std == 100.0
    assert all(c.eps == 1e-5 for c in I.CONFIGS)


def test_generator_is_seeded_and_storage_exact():
    c = I.custom("bf16", 64, 48, 80, seed=9)
    a, b = I.generate(c), I.generate(c)
    for k in a:
        assert torch.equal(a[k], b[k])
        assert torch.equal(a[k].to(torch.bfloat16).to(torch.float32), a[k]), k   # already bf16 values
    d = I.generate(I.custom("bf16", 64, 48, 80, seed=10))
    assert not torch.equal(a["X"], d["X"])
    f = I.generate(I.custom("f32", 64, 48, 80, seed=9))
    assert torch.equal(f["X"].to(torch.bfloat16).to(torch.float32), a["X"])          # same draws, then rounded


def test_distributions_follow_the_variance_reading():
    c = I.custom("f32", 2048, 256, 2048, seed=3, x_mean=50.0, x_std=100.0)
    t = I.generate(c)
    assert abs(t["X"].mean().item() - 50) < 0.5 and abs(t["X"].std().item() - 100) < 0.5
    assert abs(t["W"].std().item() - 256 ** -0.5) < 1e-3
    assert abs(t["b"].std().item() - 0.02 ** 0.5) < 0.01
    assert abs(t["gamma"].mean().item() - 1) < 0.03 and abs(t["gamma"].std().item() - 0.1 ** 0.5) < 0.02
    assert abs(t["beta"].std().item() - 0.1 ** 0.5) < 0.02
    assert abs(t["dY"].std().item() - 1) < 0.01


def test_oracle_matches_stored_tripwire():
    spec = importlib.util.spec_from_file_location("mk", os.path.join(HERE, "golden", "make_oracle_golden.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    r = O.forward_backward(**mk.case())
    with open(os.path.join(HERE, "golden", "oracle_tiny.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            k, *vals = line.split()
            np.testing.assert_allclose(np.asarray(r[k]).ravel(), np.array([float(v) for v in vals]),
                                       rtol=1e-13, atol=1e-15, err_msg=k)


def test_small_config_outputs_are_not_degenerate():
    c0 = I.CONFIGS[0]
    t = {k: v.numpy() for k, v in I.generate(c0).items()}
    r = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"], c0.eps)
    t2 = {k: v.numpy() for k, v in I.generate(I.custom("f32", c0.M, c0.K, c0.N, seed=100)).items()}
    r2 = O.forward_backward(t2["X"], t2["W"], t2["b"], t2["gamma"], t2["beta"], t2["dY"], c0.eps)
    for k in ("Y", "dX", "dW"):
        v = r[k]
        assert v.max() - v.min() > 0.02, k                       # not confined to +-0.01
        assert v.std(axis=0).min() > 1e-3 and v.std(axis=1).min() > 1e-3, k   # not uniform along an axis
        assert np.abs(v - r2[k]).max() > 0.01, k                 # depends on the inputs
