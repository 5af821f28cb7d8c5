"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares, and
rejects everything the host can check before any device work is enqueued."""
import ctypes
import os
import re

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ada():
    from paper_2605_03110_amd import ada as mod
    if not os.path.exists(mod.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return mod


def header_functions():
    text = open(os.path.join(ROOT, "include", "ada.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ada_[a-z_]+)\s*\(", text)))


def test_header_declares_the_two_calls_of_the_task_and_helpers():
    names = header_functions()
    assert "ada_select_full" in names and "ada_cascade_step" in names
    assert len(names) >= 5


def test_library_exports_every_declared_symbol(ada):
    lib = ctypes.CDLL(ada.LIB_PATH)
    for name in header_functions():
        assert hasattr(lib, name), name
    assert sorted(ada.SYMBOLS) == header_functions()


def test_binding_has_the_same_names(ada):
    import paper_2605_03110_amd as pa
    for name in header_functions():
        if name in ("ada_status_string", "ada_workspace_bytes"):
            continue
        assert hasattr(pa, name), name


def test_workspace_size_is_monotone_and_small(ada):
    assert ada.workspace_bytes(0) == 0
    sizes = [ada.workspace_bytes(T) for T in (1, 512, 2048, 8192)]
    assert sizes == sorted(sizes) and sizes[-1] < 16 << 20     # dominated by the hit table: T * T / 8 bytes
    assert all(s % 256 == 0 for s in sizes)


def test_status_strings(ada):
    seen = {ada.status_string(i) for i in range(8)}
    assert len(seen) == 8 and ada.status_string(0) == "ADA_OK"
    assert "unknown" in ada.status_string(99)


def _call_full(ada, X=0x1000, T=8, d=8, ld=8, dtype=1, tau=0.1, mask=0x1000, idx=0x1000, count=0x1000, gamma=None,
               ws=0x1000, ws_bytes=1 << 20):
    return ada.lib().ada_select_full(X, T, d, ld, dtype, tau, mask, idx, count, gamma, ws, ws_bytes, None, 0)


def _call_step(ada, X=0x1000, T=8, d=8, ld=8, dtype=1, tau=0.1, prev=0x1000, r=2, idx=0x1000, adds=0x1000,
               removes=0x1000, counts=0x1000, ws=0x1000, ws_bytes=1 << 20):
    return ada.lib().ada_cascade_step(X, T, d, ld, dtype, tau, prev, r, None, idx, adds, removes, counts, None, None,
                                      ws, ws_bytes, None, 0)


def test_host_checkable_errors_return_before_touching_the_device(ada):
    """Pointers here are never dereferenced: every case must be rejected by the argument checks."""
    NULL, SHAPE, TAU, WS, DTYPE = 1, 2, 3, 5, 7
    assert _call_full(ada, X=None) == NULL
    assert _call_full(ada, mask=None) == NULL
    assert _call_full(ada, count=None) == NULL
    assert _call_full(ada, ws=None) == NULL
    assert _call_full(ada, T=0) == SHAPE
    assert _call_full(ada, d=0) == SHAPE
    assert _call_full(ada, ld=7) == SHAPE
    assert _call_full(ada, T=(1 << 20) + 1, ws_bytes=1 << 40) == SHAPE
    assert _call_full(ada, dtype=5) == DTYPE
    for tau in (0.0, 1.0, -0.5, 2.0, float("nan")):
        assert _call_full(ada, tau=tau) == TAU
        assert _call_step(ada, tau=tau) == TAU
    assert _call_full(ada, ws_bytes=16) == WS
    assert _call_full(ada, ws=0x1010) == WS          # not 256-byte aligned
    assert _call_step(ada, prev=None) == NULL
    assert _call_step(ada, idx=None) == NULL
    assert _call_step(ada, adds=None) == NULL
    assert _call_step(ada, removes=None) == NULL
    assert _call_step(ada, counts=None) == NULL
    assert _call_step(ada, r=0) == SHAPE
    assert _call_step(ada, r=9) == SHAPE
    lib = ada.lib()

    def assign(X=0x1000, T=8, d=8, ld=8, dtype=1, idx=0x1000, r=2, out=0x1000, info=0x1000, ws=0x1000, nb=1 << 20):
        return lib.ada_assign_nearest(X, T, d, ld, dtype, idx, r, None, out, None, info, ws, nb, None, 0)
    assert assign(X=None) == NULL and assign(idx=None) == NULL and assign(out=None) == NULL
    assert assign(info=None) == NULL and assign(ws=None) == NULL
    assert assign(r=0) == SHAPE and assign(r=9) == SHAPE and assign(T=0) == SHAPE and assign(ld=7) == SHAPE
    assert assign(dtype=3) == DTYPE and assign(nb=64) == WS

    def attn(Q=0x1000, T=8, H=2, dh=64, ld=128, dtype=1, idx=0x1000, r=2, a=0x1000, out=0x1000, ldo=128, info=0x1000,
             ws=0x1000, nb=1 << 20):
        return lib.ada_attention_compressed(Q, 0x1000, 0x1000, T, H, dh, ld, dtype, idx, r, None, a, out, ldo, info,
                                            ws, nb, None, 0)
    assert attn(Q=None) == NULL and attn(idx=None) == NULL and attn(a=None) == NULL and attn(out=None) == NULL
    assert attn(info=None) == NULL and attn(ws=None) == NULL
    assert attn(dh=48) == SHAPE and attn(dh=256, dtype=0, ld=512, ldo=512) == SHAPE      # fp32 heads stop at 128
    assert attn(ld=64) == SHAPE and attn(ldo=64) == SHAPE and attn(r=0) == SHAPE and attn(r=9) == SHAPE
    assert attn(Q=0x1008) == SHAPE and attn(dtype=4) == DTYPE and attn(nb=64) == WS
    assert lib.ada_set_overlap(None, 0x1000, 4, 0x1000, None) == NULL
    assert lib.ada_set_overlap(0x1000, 0x1000, 0, 0x1000, None) == SHAPE
    ptrs = (ctypes.c_void_p * 2)(0x1000, None)
    assert lib.ada_cascade_layers(ptrs, 2, 8, 8, 8, 1, 0.1, 0x1000, 0x1000, 0x1000, None, None, 0x1000, 1 << 20,
                                  None, 0) == NULL
    assert lib.ada_cascade_layers(ptrs, 0, 8, 8, 8, 1, 0.1, 0x1000, 0x1000, 0x1000, None, None, 0x1000, 1 << 20,
                                  None, 0) == SHAPE

    def batched(X=ptrs, B=1, L=1, T=8, ws=0x1000, nb=1 << 20):
        return lib.ada_cascade_layers_batched(X, B, L, T, 8, 8, 1, 0.1, 0x1000, 0x1000, 0x1000, None, None, ws, nb,
                                              None, None, 0)
    assert batched(X=None) == NULL and batched(ws=None) == NULL and batched(B=2) == NULL      # second pointer is NULL
    assert batched(B=0) == SHAPE and batched(L=0) == SHAPE and batched(B=4097) == SHAPE and batched(T=0) == SHAPE
    one = lib.ada_workspace_bytes(8)
    two = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    assert batched(X=two, B=2, nb=2 * one - 1) == WS and batched(ws=0x1010) == WS

    import paper_2605_03110_amd as pa

    def grouped(g=(2, 8, 8, 4, 1), X=0x1000, T=8, d=8, ld=16, prev=0x1000, r=2, idx=0x1000, ws=0x1000, nb=1 << 20, nog=False):
        gs = pa.AdaGroups(*g)
        return lib.ada_cascade_step_grouped(None if nog else ctypes.byref(gs), X, T, d, ld, 1, 0.1, prev, r, None, idx,
                                            0x1000, 0x1000, 0x1000, 0x1000, ws, nb, None, 0)
    assert grouped(nog=True) == NULL and grouped(X=None) == NULL and grouped(prev=None) == NULL and grouped(ws=None) == NULL
    assert grouped(g=(0, 8, 8, 4, 1)) == SHAPE and grouped(g=(4097, 8, 8, 4, 1)) == SHAPE
    assert grouped(g=(2, 7, 8, 4, 1)) == SHAPE and grouped(g=(2, 8, 7, 4, 1)) == SHAPE       # strides below d / T
    assert grouped(g=(2, 8, 8, 3, 1)) == SHAPE and grouped(g=(2, 8, 8, 4, 0)) == SHAPE
    assert grouped(r=0) == SHAPE and grouped(r=9) == SHAPE and grouped(T=0) == SHAPE
    assert grouped(nb=2 * one - 1) == WS and grouped(ws=0x1010) == WS
    fullg = lambda g=(2, 8, 8, 4, 1), X=0x1000, idx=0x1000, ws=0x1000, nb=1 << 20: lib.ada_select_full_grouped(
        ctypes.byref(pa.AdaGroups(*g)), X, 8, 8, 16, 1, 0.1, None, idx, 0x1000, ws, nb, None, 0)
    assert fullg(X=None) == NULL and fullg(idx=None) == NULL and fullg(ws=None) == NULL
    assert fullg(g=(0, 8, 8, 4, 1)) == SHAPE and fullg(g=(2, 7, 8, 4, 1)) == SHAPE and fullg(g=(2, 8, 8, 3, 1)) == SHAPE
    assert fullg(nb=2 * one - 1) == WS
    gs = pa.AdaGroups(2, 8, 0, 0, 0)
    lay = lambda X=two, L=2, nb=1 << 20, G=gs: lib.ada_cascade_layers_grouped(
        ctypes.byref(G), X, L, 8, 8, 16, 1, 0.1, 0x1000, 0x1000, 0x1000, None, None, 0x1000, nb, None, 0)
    assert lay(X=None) == NULL and lay(X=ptrs) == NULL and lay(L=0) == SHAPE and lay(nb=2 * one - 1) == WS
    assert lay(G=pa.AdaGroups(2, 7, 0, 0, 0)) == SHAPE and lay(G=pa.AdaGroups(0, 8, 0, 0, 0)) == SHAPE

    good = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    outs = (ctypes.c_void_p * 2)(0x3000, 0x4000)

    def pipe(X=good, Q=good, outp=outs, L=2, T=8, H=2, dh=64, ld=128, dtype=1, idx=0x1000, ldo=128, ws=0x1000, nb=1 << 20):
        return lib.ada_pipeline_layers(X, Q, good, good, L, T, H, dh, ld, dtype, 0.1, idx, 0x1000, 0x1000, 0x1000, 0x1000,
                                       outp, ldo, ws, nb, None, None, None, 0)
    assert pipe(X=None) == NULL and pipe(Q=ptrs) == NULL and pipe(outp=None) == NULL and pipe(idx=None) == NULL
    assert pipe(ws=None) == NULL
    assert pipe(L=0) == SHAPE and pipe(H=0) == SHAPE and pipe(dh=48) == SHAPE and pipe(ld=64) == SHAPE and pipe(ldo=64) == SHAPE
    assert pipe(T=0) == SHAPE and pipe(dtype=5) == DTYPE
    assert pipe(nb=2 * lib.ada_workspace_bytes(8) - 1) == WS and pipe(ws=0x1010) == WS
    odd = (ctypes.c_void_p * 2)(0x1000, 0x2008)
    assert pipe(Q=odd) == SHAPE

    TAU = 3

    def adaptive(X=good, ctl=(0.1, 0.2, 0.05, 0.5), tau0=0.1, L=2, T=8, tau_all=0x1000, ws=0x1000, nb=1 << 20, flags=0, noctl=False):
        c = pa.AdaTauControl(*ctl)
        return lib.ada_cascade_layers_adaptive(X, L, T, 8, 8, 1, tau0, None if noctl else ctypes.byref(c), 0x1000, 0x1000,
                                               0x1000, None, None, tau_all, 0x1000, ws, nb, None, flags)
    assert adaptive(X=None) == NULL and adaptive(noctl=True) == NULL and adaptive(tau_all=None) == NULL and adaptive(X=ptrs) == NULL
    assert adaptive(L=0) == SHAPE and adaptive(T=0) == SHAPE and adaptive(flags=2) == SHAPE
    assert adaptive(ctl=(0.1, 0.2, 0.0, 0.5)) == TAU and adaptive(ctl=(0.1, 0.2, 0.05, 1.0)) == TAU
    assert adaptive(ctl=(0.1, 0.2, 0.3, 0.2)) == TAU and adaptive(tau0=0.6) == TAU and adaptive(tau0=0.01) == TAU
    assert adaptive(ctl=(float("nan"), 0.2, 0.05, 0.5)) == TAU and adaptive(nb=64) == WS


def test_binding_rejects_host_tensors_and_wrong_dtypes(ada):
    import paper_2605_03110_amd as pa
    with pytest.raises(ValueError):
        pa.ada_select_full(torch.zeros(4, 4), 0.1)
    with pytest.raises(ValueError):
        pa.ada_cascade_layers([], 0.1)


def test_cascade_report_is_the_papers_bookkeeping(ada):
    """Host-only entry point: Table 5's first GPT-J rows reproduce the printed turnover, and the Jaccard of
    consecutive cascade sets follows from the counts."""
    import paper_2605_03110_amd as pa
    # layer: r, adds, removes  (Table 5: 69 -> 200 -> 123 -> 164)
    counts = torch.tensor([[69, 69, 0, 0], [200, 131, 0, 0], [123, 34, 111, 0], [164, 69, 28, 0]], dtype=torch.int32)
    T = 512
    ops = torch.tensor([T * T, 69 * 69 + (T - 69) * 69, 200 * 200 + (T - 200) * 89, 123 * 123 + (T - 123) * 95],
                       dtype=torch.int64)
    rep = pa.ada_cascade_report(counts, ops, T)
    assert [round(100 * x) for x in rep["turnover"][1:]] in ([190, 72, 79], [190, 73, 79])
    assert rep["jaccard"][1] == pytest.approx(69 / 200)
    assert rep["jaccard"][2] == pytest.approx((200 - 111) / (200 + 34))
    assert rep["savings"] == pytest.approx(1 - float(ops.sum()) / (4 * T * T))


def test_tile_shape_plan_follows_tiles_per_workgroup(ada):
    """The cost model of the cascade tiles (host-side evaluation of the function the kernel uses): rounds of tiles
    per workgroup x (weighted bytes per tile + a fixed part).  The three d = 4096 configurations take three different
    shapes on a 256-CU device; sharing the device among groups pushes towards the larger tiles; short rows too."""
    lib = ada.lib()
    plan = lib.ada_plan_tile_shape
    assert plan(435, 2048, 4096, 256) == 0          # 224 tiles of 64 x 64: one round, least bytes per workgroup
    assert plan(920, 2048, 4096, 256) == 1          # 480 / 240 / 128 tiles: 64 x 128 is one round of 1.5 MB
    assert plan(690, 8192, 4096, 256) == 3          # 1408 / 704 / 384 / 192 tiles: one round of 128 representatives x 256 tokens
    assert plan(435, 2048, 4096, 64) == 2           # a quarter of the device per sequence
    assert plan(435, 2048, 256, 16) == 3            # 16 heads of 256 columns: short rows, the fixed part per round decides
    assert plan(20, 64, 4096, 256) == 0 and plan(1, 1, 1, 1) == 0
    assert plan(0, 8, 8, 8) == -1 and plan(9, 8, 8, 8) == -1 and plan(4, 8, 0, 8) == -1 and plan(4, 8, 8, 0) == -1
    for r, T, d, wg in [(300, 4096, 1024, 256), (2000, 4096, 4096, 256), (5000, 16384, 512, 128)]:
        assert plan(r, T, d, wg) in (0, 1, 2, 3)


def test_full_selection_unit_plan(ada):
    """How the full selection's direct-to-LDS kernel cuts the triangle (host-side evaluation of the launch's own
    choice): halved units where 128 x 128 units leave CUs idle, 128 x 128 units where they fill the chip in whole
    rounds, 256 x 256 units beyond the one-launch form's range."""
    plan = ada.lib().ada_plan_full_units
    assert plan(2048, 4096, 256) == 2               # 240 + 16 = 256 units on 256 CUs instead of 136 of 128 x 128
    assert plan(1536, 4096, 256) == 2               # 144 instead of 78
    assert plan(2560, 4096, 256) == 0               # 210 units of 128 x 128 in one round; halved ones would take two
    assert plan(4096, 4096, 256) == 0
    assert plan(2048, 4096 + 32, 256) in (0, 1)     # rows in half chunks: not the one-launch form
    assert plan(8192, 4096, 256) == 1               # 496 units of 256 x 256 and the diagonal in 128 x 128 units
    assert plan(1535, 4096, 256) == -1 and plan(2048, 48, 256) == -1 and plan(2048, 4096, 4) == -1
    assert plan(1 << 30, 4096, 256) == -1


def test_build_reads_the_compilers_resource_report(ada):
    """The build refuses a hot kernel that needs more private (scratch) memory than its budget; here only the reading of
    the compiler's remarks is checked (the build itself runs them on every compile)."""
    remarks = (
        "a.hpp:10:1: remark: Function Name: _ZN1x15k_cascade_fusedItLb1ELi2ELb1EEEv [-Rpass-analysis=kernel-resource-usage]\n"
        "   10 | __global__ void k() {\n      | ^\n"
        "a.hpp:10:1: remark:     TotalSGPRs: 104 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hpp:10:1: remark:     VGPRs: 239 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hpp:10:1: remark:     ScratchSize [bytes/lane]: 20 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hpp:10:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]\n"
        "b.hpp:20:1: remark: Function Name: _ZN1x10k_gram_dmaILb1EEEv [-Rpass-analysis=kernel-resource-usage]\n"
        "b.hpp:20:1: remark:     VGPRs: 169 [-Rpass-analysis=kernel-resource-usage]\n"
        "b.hpp:20:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n")
    got = ada.kernel_resources(remarks)
    assert got["_ZN1x15k_cascade_fusedItLb1ELi2ELb1EEEv"] == {"TotalSGPRs": 104, "VGPRs": 239, "ScratchSize": 20}
    assert got["_ZN1x10k_gram_dmaILb1EEEv"] == {"VGPRs": 169, "ScratchSize": 0}
    assert all(isinstance(v, int) and v >= 0 for v in ada.SCRATCH_BUDGET.values())
