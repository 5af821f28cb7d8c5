"""ada_cascade_step_static (the entry point for callers that cannot allocate) against ada_cascade_step: same
kernels, scratch memory in the library's own image instead of a caller's workspace.  Two calls in a row, the second
on a smaller input, each compared bit for bit with the workspace form and step by step with the oracle.  Runs last
(the file name sorts behind the other GPU tests) and passes alone in a fresh process as well."""
import os
import sys

import numpy as np
import pytest
import torch

import paper_2605_03110_amd as pa
from paper_2605_03110_amd import workloads as wl

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def both_forms(w, flags):
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    full = pa.fetch(pa.ada_select_full(xs[0], w.tau))
    prev = torch.from_numpy(full["idx"]).to(DEV)
    want = pa.ada_cascade_step(xs[1], w.tau, prev, flags=flags)
    # the caller's own output tensors, allocated before the call that must not allocate; poisoned so that a call
    # that wrote nothing cannot pass
    out = {k: torch.full_like(v, -1) for k, v in want.items() if isinstance(v, torch.Tensor)}
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    pa.ada_cascade_step_static(xs[1], w.tau, prev, out, flags=flags)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # nothing came from torch's allocator
    a, b = pa.fetch(want), pa.fetch(out)
    for k in ("idx", "adds", "removes"):
        assert np.array_equal(a[k], b[k]), k
    assert (a["r"], a["n_adds"], a["n_removes"], a["gram_ops"]) == (b["r"], b["n_adds"], b["n_removes"], b["gram_ops"])
    assert np.array_equal(a["gamma"], b["gamma"])             # same kernels, same arithmetic: identical bits
    parity.check_cascade(xs_cpu[1], w.tau, full["idx"], b, what=w.name, two_pass=bool(flags & pa.FLAG_TWO_PASS))
    return b


@pytest.mark.parametrize("flags", [0, pa.FLAG_TWO_PASS])
def test_static_scratch_matches_the_workspace_form_on_two_calls_in_a_row(flags):
    print("[case] no-alloc entry point, flags %d" % flags, flush=True)
    big = both_forms(wl.small(T=pa.STATIC_MAX_T, d=256, K=500, L=2, dtype="bf16", seed=31, p=0.08), flags)   # the largest T it takes
    small = both_forms(wl.small(T=333, d=200, K=40, L=2, dtype="bf16", seed=32, p=0.1), flags)   # reuses the array
    assert big["r"] > small["r"] > 0
    both_forms(wl.small(T=300, d=96, K=40, L=2, dtype="f32", seed=33, p=0.1), flags)


def test_static_scratch_rejects_what_does_not_fit():
    T = pa.STATIC_MAX_T + 1
    x = torch.zeros((T, 64), dtype=torch.bfloat16, device=DEV)
    prev = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = dict(idx=torch.empty(T, dtype=torch.int32, device=DEV), adds=torch.empty(T, dtype=torch.int32, device=DEV),
               removes=torch.empty(1, dtype=torch.int32, device=DEV), counts=torch.empty(4, dtype=torch.int32, device=DEV),
               gram_ops=torch.empty(1, dtype=torch.int64, device=DEV), gamma=torch.empty(T, dtype=torch.float32, device=DEV))
    with pytest.raises(pa.AdaError) as e:
        pa.ada_cascade_step_static(x, 0.1, prev, out)
    assert e.value.status == 2          # ADA_ERR_SHAPE, reported before anything is enqueued
