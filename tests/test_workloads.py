"""The seeded input generator: determinism, shapes, dtypes and the regime each
scale reading produces (checked with the oracle)."""
import numpy as np
import torch

import oracle
from paper_2605_03110_amd import workloads as wl


def test_five_configs_have_the_stated_shapes():
    shapes = [(w.T, w.d, w.L, w.dtype, w.K, w.batch) for w in wl.CONFIGS]
    assert shapes == [(512, 768, 12, "f32", 100, 1), (2048, 768, 12, "bf16", 400, 1),
                      (2048, 4096, 28, "bf16", 400, 1), (2048, 4096, 32, "bf16", 1000, 1),
                      (8192, 4096, 32, "bf16", 400, 4)]
    assert all(w.tau == 0.1 for w in wl.CONFIGS)


def test_generator_is_deterministic_and_sequences_differ():
    w = wl.small(T=64, d=40, K=8, L=3)
    a, b = wl.layer_list(w, 0), wl.layer_list(w, 0)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    c = wl.layer_list(w, 1)
    assert not torch.equal(a[0], c[0])
    assert a[0].dtype == torch.bfloat16 and tuple(a[0].shape) == (64, 40)
    assert wl.layer_list(wl.small(T=8, d=4, K=2, L=1, dtype="f32"))[0].dtype == torch.float32


def test_bf16_values_widen_exactly():
    x = wl.layer_list(wl.small(T=16, d=24, K=4, L=1))[0]
    assert np.array_equal(wl.as_f64(x), x.to(torch.float32).numpy().astype(np.float64))


def test_relative_scale_makes_same_centre_tokens_redundant_and_literal_does_not():
    # literal noise energy d * 0.004^2 must exceed tau^2 = 0.01 for same-centre cosines to drop below 0.99
    rel = wl.small(T=200, d=2048, K=20, L=1, dtype="f32", seed=5)
    lit = wl.small(T=200, d=2048, K=20, L=1, dtype="f32", seed=5, scale="literal")
    r_rel = oracle.select_full(wl.as_f64(wl.layer_list(rel)[0]), rel.tau)["r"]
    r_lit = oracle.select_full(wl.as_f64(wl.layer_list(lit)[0]), lit.tau)["r"]
    assert r_rel <= 20
    assert r_lit == 200


def test_reassignment_drives_turnover():
    w = wl.small(T=300, d=64, K=30, L=4, dtype="f32", seed=9, p=0.1)
    Xs = [wl.as_f64(x) for x in wl.layer_list(w)]
    R = oracle.select_full(Xs[0], w.tau)["idx"]
    changed = 0
    for X in Xs[1:]:
        res = oracle.cascade_step(X, w.tau, R)
        changed += len(res["adds"]) + len(res["removes"])
        R = res["idx"]
    assert changed > 0
