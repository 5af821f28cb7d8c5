"""Parity of the HIP path (through the C ABI) against the float64 oracle on the same seeded inputs."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2605_03110_amd as pa
from paper_2605_03110_amd import workloads as wl

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(autouse=True)
def dev_switches(monkeypatch):
    """the library reads its path-forcing variables only under this master switch"""
    monkeypatch.setenv("ADA_DEV_SWITCHES", "1")


def say(msg):
    print("[case] " + msg, flush=True)


def dev_idx(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.int32))).to(DEV)


def oflags(flags):
    """library flags -> oracle flags (the oracle knows only the cross-step reading)"""
    return oracle.CROSS_EARLIER_ONLY if flags & pa.FLAG_CROSS_EARLIER_ONLY else 0


def step_and_check(x_dev, x_cpu, tau, prev, flags=0, what="", **kw):
    got = pa.fetch(pa.ada_cascade_step(x_dev, tau, dev_idx(prev), flags=flags, **kw))
    info = parity.check_cascade(x_cpu, tau, prev, got, flags=oflags(flags), what=what,
                                two_pass=bool(flags & pa.FLAG_TWO_PASS))
    return got, info


def run_layers_teacher_forced(w, xs_cpu, flags=0, what=""):
    """full at layer 0, then a cascade step per layer on the GPU's own previous output; oracle checks each."""
    xs = [x.to(DEV) for x in xs_cpu]
    full = pa.fetch(pa.ada_select_full(xs[0], w.tau))
    parity.check_full(xs_cpu[0], w.tau, full, what + " layer 0")
    prev = full["idx"]
    stats = []
    for l in range(1, len(xs)):
        got, info = step_and_check(xs[l], xs_cpu[l], w.tau, prev, flags, "%s layer %d" % (what, l))
        stats.append((got["n_adds"], got["n_removes"], info["gamma_err"]))
        prev = got["idx"]
    return stats


# ------------------------------------------------------------------------------------------ small shapes
SMALL = [
    # T, d, K, dtype
    (1, 16, 1, "bf16"),
    (2, 8, 1, "f32"),
    (63, 64, 9, "bf16"),
    (64, 64, 9, "f32"),
    (130, 72, 17, "f32"),
    (333, 200, 40, "bf16"),
    (257, 1030, 33, "bf16"),     # d not a multiple of 8: element-wise loader, ragged K chunk
    (200, 37, 21, "f32"),        # d not a multiple of 4
    (513, 768, 100, "f32"),
    (700, 4096, 120, "bf16"),
]


@pytest.mark.parametrize("tile", ["64", "128"])
@pytest.mark.parametrize("T,d,K,dtype", SMALL)
def test_small_shapes_full_and_two_launch_cascade(T, d, K, dtype, tile, monkeypatch):
    monkeypatch.setenv("ADA_TILE", tile)
    say("small T=%d d=%d K=%d %s tile=%s two-launch" % (T, d, K, dtype, tile))
    w = wl.small(T=T, d=d, K=K, L=3, dtype=dtype, seed=17 + T, p=0.1)
    stats = run_layers_teacher_forced(w, wl.layer_list(w), flags=pa.FLAG_TWO_PASS, what="small T=%d d=%d" % (T, d))
    assert all(e <= parity.GAMMA_TOL for _, _, e in stats)


@pytest.mark.parametrize("kgroups", ["1", "2"])
@pytest.mark.parametrize("T,d,K,dtype", SMALL)
def test_small_shapes_one_launch_cascade(T, d, K, dtype, kgroups, monkeypatch):
    monkeypatch.setenv("ADA_KGROUPS", kgroups)
    say("small T=%d d=%d K=%d %s one-launch kgroups=%s" % (T, d, K, dtype, kgroups))
    w = wl.small(T=T, d=d, K=K, L=3, dtype=dtype, seed=17 + T, p=0.1)
    stats = run_layers_teacher_forced(w, wl.layer_list(w), what="small T=%d d=%d" % (T, d))
    assert all(e <= parity.GAMMA_TOL for _, _, e in stats)


@pytest.mark.parametrize("tile", ["64x128", "128", "256x128"])
@pytest.mark.parametrize("T,d,K,dtype", [(1, 64, 1, "bf16"), (130, 64, 17, "bf16"), (333, 192, 40, "bf16"), (300, 96, 40, "f32"),
                                         (700, 4096, 120, "bf16"), (1290, 128, 300, "bf16"), (2100, 320, 700, "bf16")])
def test_small_shapes_one_launch_cascade_on_wide_tiles(T, d, K, dtype, tile, monkeypatch):
    """The wide tiles of the one-launch cascade (rows in whole aligned 128-byte chunks: 64 x 128 on the 128-byte-chunk
    ring; 128 x 128 and 128 representatives x 256 tokens on the half-chunk ring for bf16), forced onto small and ragged
    shapes; the assignment runs on the same tiles."""
    monkeypatch.setenv("ADA_CASCADE_TILE", tile)
    say("small T=%d d=%d K=%d %s one-launch, %s tiles" % (T, d, K, dtype, tile))
    w = wl.small(T=T, d=d, K=K, L=3, dtype=dtype, seed=23 + T, p=0.1)
    xs = wl.layer_list(w)
    stats = run_layers_teacher_forced(w, xs, what="%s tiles T=%d d=%d" % (tile, T, d))
    assert all(e <= parity.GAMMA_TOL for _, _, e in stats)
    run_layers_teacher_forced(w, xs, flags=pa.FLAG_CROSS_EARLIER_ONLY, what="%s tiles earlier-only T=%d" % (tile, T))
    full = pa.fetch(pa.ada_select_full(xs[0].to(DEV), w.tau))
    res = pa.ada_assign_nearest(xs[0].to(DEV), torch.as_tensor(full["idx"]).to(DEV))
    parity.check_assign(xs[0], full["idx"], res["assign"].cpu().numpy(), res["corr"].cpu().numpy(), "%s tiles assign" % tile)


@pytest.mark.parametrize("path", ["dma0", "dma1", "dma2"])
@pytest.mark.parametrize("T,d,K", [(257, 128, 30), (700, 4096, 120), (1000, 64, 90), (1, 64, 1), (129, 32, 8),
                                   (1290, 96, 140), (512, 160, 60), (3000, 64, 300), (5500, 32, 400),
                                   (4096, 64, 350), (4097, 64, 350)])
def test_direct_to_lds_full_selection(T, d, K, path, monkeypatch):
    """The direct-to-LDS Gram kernel of the full selection, every way of cutting the triangle into units (128 x 128
    everywhere; 256 x 256 off the diagonal, which the one-launch form up to T = 4096 does not have; 64 x 128 off the
    diagonal with the diagonal blocks' rows staged once, which only that form has), forced onto small and ragged shapes (T off the 128 and 256 grids, one to three half chunks, a single token) and onto
    shapes with more units than workgroups, where the rest is handed out through the counter in the workspace.
    Up to T = 4096 the kernel's last workgroup applies the threshold and compacts the set; beyond (4097, 5500) the
    update is a launch of its own."""
    monkeypatch.setenv("ADA_GRAM", path)
    say("direct-to-LDS %s T=%d d=%d" % (path, T, d))
    w = wl.small(T=T, d=d, K=K, L=2, dtype="bf16", seed=29 + T, p=0.1)
    ws = pa.workspace(T, DEV)
    for x_cpu in wl.layer_list(w):
        parity.check_full(x_cpu, w.tau, pa.fetch(pa.ada_select_full(x_cpu.to(DEV), w.tau, ws=ws)), "%s T=%d" % (path, T))
    # the counters in the workspace (behind three T-word arrays and one T-byte array, each padded to 256 bytes) must
    # be back at zero for the next launch
    up = lambda n: (n + 255) // 256 * 256
    meta = ws[3 * up(4 * T) + up(T):][:2048].view(torch.int32).cpu().tolist()
    assert meta[4:7] == [0, 0, 0]
    assert [meta[4 + 64 + 32 * x] for x in range(8)] == [0] * 8          # the sign-off counters of the eight XCDs


@pytest.mark.parametrize("T,d,K,dtype", [(1600, 64, 200, "bf16"), (1600, 72, 200, "bf16"), (1600, 64, 200, "f32")])
def test_full_selection_path_choice(T, d, K, dtype):
    """Default path choice around its boundaries: the direct-to-LDS kernel (bf16, whole 64-byte pieces, T >= 1536)
    and the register-staged tile kernel next to it (d off the grid, fp32)."""
    say("path choice T=%d d=%d %s" % (T, d, dtype))
    w = wl.small(T=T, d=d, K=K, L=1, dtype=dtype, seed=41 + d, p=0.1)
    x_cpu = wl.layer_list(w)[0]
    parity.check_full(x_cpu, w.tau, pa.fetch(pa.ada_select_full(x_cpu.to(DEV), w.tau)), "path choice")


def test_default_tile_heuristic_runs_both_sizes():
    for T, d in [(300, 128), (2048, 256)]:
        say("heuristic T=%d d=%d" % (T, d))
        w = wl.small(T=T, d=d, K=50, L=2, dtype="bf16", seed=5, p=0.08)
        run_layers_teacher_forced(w, wl.layer_list(w), what="heuristic T=%d" % T)


def test_earlier_only_flag():
    say("earlier-only flag")
    w = wl.small(T=400, d=96, K=45, L=4, dtype="bf16", seed=23, p=0.15)
    xs_cpu = wl.layer_list(w)
    for extra in (0, pa.FLAG_TWO_PASS):
        run_layers_teacher_forced(w, xs_cpu, flags=extra, what="unordered")
        run_layers_teacher_forced(w, xs_cpu, flags=extra | pa.FLAG_CROSS_EARLIER_ONLY, what="earlier-only")
        # the reading-specific pin: a non-inherited duplicate of a LATER inherited token
        X = torch.tensor([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 1.0, 1e-3, 0]], dtype=torch.float32)
        prev = [0, 2]
        g0, _ = step_and_check(X.to(DEV), X, 0.1, prev, extra)
        g1, _ = step_and_check(X.to(DEV), X, 0.1, prev, extra | pa.FLAG_CROSS_EARLIER_ONLY)
        assert g0["idx"].tolist() == [0, 2] and g1["idx"].tolist() == [0, 1, 2]


# ------------------------------------------------------------------------------------------ edge cases
def test_extreme_inherited_sets():
    w = wl.small(T=150, d=80, K=12, L=2, dtype="bf16", seed=41)
    xs_cpu = wl.layer_list(w)
    x = xs_cpu[1].to(DEV)
    for prev in ([0], [149], list(range(150)), list(range(0, 150, 2)), [3, 77]):
        say("extreme inherited set of size %d" % len(prev))
        for flags in (0, pa.FLAG_TWO_PASS):
            step_and_check(x, xs_cpu[1], w.tau, prev, flags, "prev size %d" % len(prev))


@pytest.mark.parametrize("T,d,dtype", [(256, 128, "bf16"), (1024, 256, "f32"), (4096, 512, "bf16"), (2052, 192, "bf16")])
def test_chains_whose_earliest_hit_is_a_removed_representative(T, d, dtype):
    """Chains t ~ s1 ~ s0 with t not ~ s0 (Algorithm 1 steps 5 and 9): s1 is removed because the earlier s0 hits it, so
    the earliest representative that hits t does not count, and t is covered only where a later, valid s2 hits it too.
    Each group of four tokens lives in its own plane: s0 at 0, s1 at 7, t at 13 and (every other group) s2 at 18
    degrees, far from the threshold angle of 8.1 degrees; the groups' tokens are interleaved in several orders."""
    say("chains through removed representatives, T=%d d=%d %s" % (T, d, dtype))
    rng = np.random.default_rng(T + d)
    G = min(d // 2, T // 4)
    X = np.zeros((T, d), dtype=np.float32)
    ang = np.deg2rad([0.0, 7.0, 13.0, 18.0])
    slots = rng.permutation(T)[:4 * G].reshape(G, 4)
    inherited = []
    for g in range(G):
        ids = np.sort(slots[g])
        t_at = int(rng.integers(0, 4))                       # where the chain's tail sits among the group's token ids
        s_ids = [i for k, i in enumerate(ids) if k != t_at]  # s0 < s1 < s2 in token order
        t_id = ids[t_at]
        scale = rng.uniform(0.5, 2.0, size=4)                # norms must not matter
        for a, tok, sc in zip(ang[[0, 1, 3]], s_ids, scale[:3]):
            X[tok, 2 * g], X[tok, 2 * g + 1] = sc * np.cos(a), sc * np.sin(a)
        X[t_id, 2 * g], X[t_id, 2 * g + 1] = scale[3] * np.cos(ang[2]), scale[3] * np.sin(ang[2])
        inherited += s_ids[:2] + (s_ids[2:] if g % 2 == 0 else [])
        if g % 2 == 1:                                       # no s2 in R: its row becomes one more tail of the chain s1
            X[s_ids[2], 2 * g], X[s_ids[2], 2 * g + 1] = np.cos(ang[2]), -np.sin(ang[2])   # 20 degrees from s1: alone
    x_cpu = wl.to_dtype(X, dtype)
    prev = np.sort(np.asarray(inherited, dtype=np.int32))
    for flags in (0, pa.FLAG_TWO_PASS):
        got, info = step_and_check(x_cpu.to(DEV), x_cpu, 0.1, prev, flags, "chains flags %d" % flags)
        assert info["n_band"] == 0
        assert got["n_removes"] == G                          # every s1
        assert G // 2 <= got["n_adds"]                        # every tail without a valid later representative


def test_duplicates_orthogonal_zero_rows_and_sign():
    say("duplicates / orthogonal / zero rows")
    rng = np.random.default_rng(3)
    base = rng.standard_normal((6, 48)).astype(np.float32)
    order = [0, 1, 0, 2, 1, 1, 3, 0, 4, 4, 2, 5]
    X = base[order] * rng.uniform(0.5, 2.0, size=(len(order), 1)).astype(np.float32)
    X[7] = -X[7]
    for dtype in ("f32", "bf16"):
        x = wl.to_dtype(X if dtype == "f32" else base[order], dtype)      # bf16: exact copies stay exact copies
        got = pa.fetch(pa.ada_select_full(x.to(DEV), 0.1))
        assert got["idx"].tolist() == [0, 1, 3, 6, 8, 11]
        parity.check_full(x, 0.1, got, "duplicates " + dtype)
    Q, _ = np.linalg.qr(rng.standard_normal((64, 64)))
    xq = wl.to_dtype((Q[:40] * 3.0).astype(np.float32), "f32")
    got = pa.fetch(pa.ada_select_full(xq.to(DEV), 0.1))
    assert got["r"] == 40
    parity.check_full(xq, 0.1, got, "orthogonal")
    Z = np.zeros((5, 16), dtype=np.float32)
    Z[1, 0] = 1.0
    Z[3, 0] = 2.0
    xz = wl.to_dtype(Z, "bf16")
    got = pa.fetch(pa.ada_select_full(xz.to(DEV), 0.1))
    assert got["mask"].tolist() == [1, 1, 1, 0, 1]
    parity.check_full(xz, 0.1, got, "zero rows")
    for flags in (0, pa.FLAG_TWO_PASS):
        step_and_check(xz.to(DEV), xz, 0.1, [0, 1, 3], flags, "zero rows cascade")


@pytest.mark.parametrize("delta", [1e-6, 1e-5, 1e-4, 1e-3])
def test_pairs_placed_around_the_threshold(delta):
    """Pairs at cos = (1 - tau^2) -/+ delta: inside the band either decision is accepted (and then forced into
    the oracle); outside it the decision must be the oracle's."""
    say("near-threshold delta=%g" % delta)
    tau = 0.1
    thr = 1 - tau * tau
    rows = []
    for sgn in (+1, -1):
        c = thr + sgn * delta
        th = np.arccos(c)
        for k in range(8 if sgn > 0 else 16)[-8:]:   # 16 unrelated planes so pairs do not interact
            a = np.zeros(64)
            b = np.zeros(64)
            a[2 * k] = 1.0
            b[2 * k] = np.cos(th)
            b[2 * k + 1] = np.sin(th)
            rows += [(a, b)]
    X = np.array([v for pair in rows for v in pair], dtype=np.float32) * 3.0
    x = wl.to_dtype(X, "f32")
    got = pa.fetch(pa.ada_select_full(x.to(DEV), tau))
    info = parity.check_full(x, tau, got, "near-threshold")
    if delta >= 1e-3:
        assert info["n_band"] == 0
        assert got["mask"].reshape(-1, 2)[:, 1].tolist() == [0] * 8 + [1] * 8
    for flags in (0, pa.FLAG_TWO_PASS):
        step_and_check(x.to(DEV), x, tau, list(range(0, 32, 2)), flags, "near-threshold cascade")
        step_and_check(x.to(DEV), x, tau, list(range(32)), flags, "near-threshold rep validation")


def test_strided_rows_and_unaligned_base():
    say("strided rows / unaligned base")
    w = wl.small(T=140, d=96, K=15, L=2, dtype="bf16", seed=51)
    xs_cpu = wl.layer_list(w)
    big = torch.zeros((140, 160), dtype=torch.bfloat16, device=DEV)
    big[:, 8:104] = xs_cpu[0].to(DEV)
    view = big[:, 8:104]                         # ld = 160 > d, 16-byte aligned base
    got = pa.fetch(pa.ada_select_full(view, w.tau))
    parity.check_full(xs_cpu[0], w.tau, got, "strided")
    big[:, 9:105] = xs_cpu[1].to(DEV)
    view = big[:, 9:105]                         # base offset 18 bytes: element-wise loader
    got = pa.fetch(pa.ada_select_full(view, w.tau))
    parity.check_full(xs_cpu[1], w.tau, got, "unaligned")


def test_bad_inherited_list_is_reported_by_the_device_and_nothing_faults():
    w = wl.small(T=100, d=64, K=10, L=1, dtype="bf16", seed=61)
    x = wl.layer_list(w)[0].to(DEV)
    ws = pa.workspace(w.T, DEV)
    for flags in (0, pa.FLAG_TWO_PASS):
        for prev in ([5, 5, 9], [9, 5], [0, 100], [-1, 3], [2**30, 2**30 + 1]):
            say("bad prev_idx %s flags=%d" % (prev[:3], flags))
            res = pa.ada_cascade_step(x, w.tau, dev_idx(prev), flags=flags, ws=ws)
            counts = res["counts"].cpu().tolist()
            assert counts[:3] == [0, 0, 0] and counts[3] == 4          # ADA_ERR_INDEX
            with pytest.raises(pa.AdaError):
                pa.fetch(res)
        r_dev = torch.tensor([0], dtype=torch.int32, device=DEV)
        res = pa.ada_cascade_step(x, w.tau, dev_idx([1, 2, 3]), r=3, r_dev=r_dev, flags=flags, ws=ws)
        assert res["counts"].cpu().tolist() == [0, 0, 0, 2]            # ADA_ERR_SHAPE: empty inherited set
        r_dev = torch.tensor([7], dtype=torch.int32, device=DEV)
        res = pa.ada_cascade_step(x, w.tau, dev_idx([1, 2, 3]), r=3, r_dev=r_dev, flags=flags, ws=ws)
        assert res["counts"].cpu().tolist()[3] == 2                    # device count beyond the list capacity
        # the workspace is left usable after a rejected list
        xs_cpu = wl.layer_list(w)
        step_and_check(x, xs_cpu[0], w.tau, [0, 7, 50], flags, "after a rejected list", ws=ws)


def test_device_side_count_and_reused_workspace():
    say("r_dev chaining")
    w = wl.small(T=500, d=128, K=60, L=3, dtype="bf16", seed=71, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    ws = pa.workspace(w.T, DEV)
    full = pa.ada_select_full(xs[0], w.tau, ws=ws)
    step = pa.ada_cascade_step(xs[1], w.tau, full["idx"], r=w.T, r_dev=full["counts"], ws=ws)   # no host sync in between
    f, s = pa.fetch(full), pa.fetch(step)
    parity.check_full(xs_cpu[0], w.tau, f)
    parity.check_cascade(xs_cpu[1], w.tau, f["idx"], s)
    step2 = pa.ada_cascade_step(xs[2], w.tau, step["idx"], r=w.T, r_dev=step["counts"], ws=ws, flags=pa.FLAG_TWO_PASS)
    parity.check_cascade(xs_cpu[2], w.tau, s["idx"], pa.fetch(step2), two_pass=True)
    raw = torch.full((pa.workspace_bytes(w.T),), 0xAB, dtype=torch.uint8, device=DEV)   # dirty memory must be initialised
    pa.ada_workspace_init(raw)
    step3 = pa.ada_cascade_step(xs[1], w.tau, full["idx"], r=w.T, r_dev=full["counts"], ws=raw)
    parity.check_cascade(xs_cpu[1], w.tau, f["idx"], pa.fetch(step3))


def test_layer_driver_matches_step_by_step_and_report():
    say("ada_cascade_layers")
    w = wl.small(T=600, d=160, K=70, L=6, dtype="bf16", seed=81, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    out = pa.ada_cascade_layers(xs, w.tau)
    torch.cuda.synchronize()
    counts = out["counts"].cpu()
    ops = out["gram_ops"].cpu()
    assert counts[:, 3].tolist() == [0] * w.L
    prev = None
    for l in range(w.L):
        r = int(counts[l, 0])
        idx = out["idx"][l, :r].cpu().numpy()
        if l == 0:
            ref = oracle.select_full(wl.as_f64(xs_cpu[0]), w.tau)
            assert np.array_equal(idx, ref["idx"]) and int(ops[0]) == w.T * w.T
        else:
            got = dict(idx=idx, adds=out["adds"][l, :int(counts[l, 1])].cpu().numpy(),
                       removes=out["removes"][l, :int(counts[l, 2])].cpu().numpy(), gram_ops=int(ops[l]),
                       r=r, n_adds=int(counts[l, 1]), n_removes=int(counts[l, 2]),
                       gamma=pa.fetch(pa.ada_cascade_step(xs[l], w.tau, dev_idx(prev)))["gamma"])
            parity.check_cascade(xs_cpu[l], w.tau, prev, got, what="driver layer %d" % l)
        prev = idx
    rep = pa.ada_cascade_report(counts, ops, w.T)
    sets = [out["idx"][l, :int(counts[l, 0])].cpu().numpy() for l in range(w.L)]
    for l in range(1, w.L):
        assert rep["jaccard"][l] == pytest.approx(oracle.metrics.jaccard(sets[l - 1], sets[l]), abs=1e-12)
        assert rep["turnover"][l] == pytest.approx(
            oracle.metrics.turnover(int(counts[l, 1]), int(counts[l, 2]), int(counts[l - 1, 0])), abs=1e-12)
    assert rep["savings"] == pytest.approx(oracle.metrics.gram_savings(ops.tolist(), w.T), abs=1e-12)
    # without the add / remove lists
    out2 = pa.ada_cascade_layers(xs, w.tau, want_lists=False)
    torch.cuda.synchronize()
    assert torch.equal(out2["counts"], out["counts"]) and torch.equal(out2["gram_ops"], out["gram_ops"])


@pytest.mark.parametrize("T,d,K,L,dtype,B", [(600, 192, 70, 5, "bf16", 3), (333, 96, 40, 4, "f32", 2),
                                             (2048, 512, 400, 4, "bf16", 4)])
def test_batched_layer_loop_on_streams(T, d, K, L, dtype, B):
    """B sequences with different seeds through ada_cascade_layers_batched, on B streams and on one stream: every
    sequence's sets, counts and lists equal those of its own ada_cascade_layers run, and every step is checked against
    the oracle on the set it consumed.  Work enqueued on the caller's stream afterwards sees the results (the copy
    below is not preceded by a device synchronisation)."""
    say("batched layer loop T=%d d=%d L=%d B=%d %s" % (T, d, L, B, dtype))
    w = wl.small(T=T, d=d, K=K, L=L, dtype=dtype, seed=91 + T, p=0.1)
    seqs_cpu = [wl.layer_list(w, sequence=b) for b in range(B)]
    seqs = [[x.to(DEV) for x in s] for s in seqs_cpu]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(B)]
    ws = pa.workspace_batched(T, B, DEV)
    for use in (streams, None, streams):                       # the third run reuses the workspaces
        out = pa.ada_cascade_layers_batched(seqs, w.tau, want_lists=True, ws=ws, streams=use)
        counts = out["counts"].to("cpu", non_blocking=False)    # on the caller's stream: joined with every chain
        idx_all, ops = out["idx"].cpu(), out["gram_ops"].cpu()
        adds_all, rem_all = out["adds"].cpu(), out["removes"].cpu()
        assert counts[:, :, 3].flatten().tolist() == [0] * (B * L)
        for b in range(B):
            single = run_driver(seqs[b], w.tau)
            sc = single["counts"].cpu()
            assert torch.equal(sc, counts[b]) and torch.equal(single["gram_ops"].cpu(), ops[b])
            for l in range(L):
                r, na, nr = (int(v) for v in sc[l, :3])
                assert torch.equal(single["idx"][l, :r].cpu(), idx_all[b, l, :r])
                if l > 0:
                    assert torch.equal(single["adds"][l, :na].cpu(), adds_all[b, l, :na])
                    assert torch.equal(single["removes"][l, :nr].cpu(), rem_all[b, l, :nr])
    first = [idx_all[b, 0, :int(counts[b, 0, 0])].tolist() for b in range(B)]
    assert first[0] != first[1]                                 # the sequences really differ
    for b in range(B):                                          # against the oracle, teacher-forced
        prev = None
        for l in range(L):
            r, na, nr = (int(v) for v in counts[b, l, :3])
            idx = idx_all[b, l, :r].numpy()
            if l == 0:
                ref = oracle.select_full(wl.as_f64(seqs_cpu[b][0]), w.tau)
                assert np.array_equal(idx, ref["idx"]) and int(ops[b, 0]) == T * T
            else:
                got = dict(idx=idx, adds=adds_all[b, l, :na].numpy(), removes=rem_all[b, l, :nr].numpy(),
                           gram_ops=int(ops[b, l]), r=r, n_adds=na, n_removes=nr,
                           gamma=pa.fetch(pa.ada_cascade_step(seqs[b][l], w.tau, dev_idx(prev)))["gamma"])
                parity.check_cascade(seqs_cpu[b][l], w.tau, prev, got, what="batched seq %d layer %d" % (b, l))
            prev = idx


@pytest.mark.parametrize("T,d,H,K,L,dtype", [(600, 512, 4, 70, 4, "bf16"), (333, 192, 3, 40, 3, "f32"), (1100, 384, 6, 150, 3, "bf16")])
def test_per_head_cascade_through_the_batched_call(T, d, H, K, L, dtype):
    """One representative set per head (Section 8.5): head h selects on the columns [h d_h, (h+1) d_h) of X, passed as
    a view (pointer offset, leading dimension d).  The H heads go through the batched layer loop as H sequences; each
    head is checked step by step against the oracle on its own column block."""
    say("per-head cascade T=%d d=%d H=%d %s" % (T, d, H, dtype))
    w = wl.small(T=T, d=d, K=K, L=L, dtype=dtype, seed=57 + T, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    dh = d // H
    heads = [[x[:, h * dh:(h + 1) * dh] for x in xs] for h in range(H)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    out = pa.ada_cascade_layers_batched(heads, w.tau, want_lists=True, streams=[streams[h % 2] for h in range(H)])
    counts = out["counts"].cpu()
    idx_all, ops, adds_all, rem_all = out["idx"].cpu(), out["gram_ops"].cpu(), out["adds"].cpu(), out["removes"].cpu()
    assert counts[:, :, 3].flatten().tolist() == [0] * (H * L)
    for h in range(H):
        prev = None
        for l in range(L):
            xh = xs_cpu[l][:, h * dh:(h + 1) * dh].contiguous()
            r, na, nr = (int(v) for v in counts[h, l, :3])
            idx = idx_all[h, l, :r].numpy()
            if l == 0:
                ref = oracle.select_full(wl.as_f64(xh), w.tau)
                assert np.array_equal(idx, ref["idx"]) and int(ops[h, 0]) == T * T
            else:
                got = dict(idx=idx, adds=adds_all[h, l, :na].numpy(), removes=rem_all[h, l, :nr].numpy(),
                           gram_ops=int(ops[h, l]), r=r, n_adds=na, n_removes=nr,
                           gamma=pa.fetch(pa.ada_cascade_step(heads[h][l], w.tau, dev_idx(prev)))["gamma"])
                parity.check_cascade(xh, w.tau, prev, got, what="head %d layer %d" % (h, l))
            prev = idx


@pytest.mark.parametrize("T,d,H,K,L,dtype", [(600, 512, 4, 70, 4, "bf16"), (333, 192, 3, 40, 3, "f32"), (1100, 384, 6, 150, 3, "bf16"),
                                             (700, 300, 6, 90, 3, "bf16"), (2048, 2048, 16, 400, 3, "bf16")])
def test_per_head_cascade_in_one_launch_per_layer(T, d, H, K, L, dtype):
    """ada_cascade_layers_grouped on the heads of one matrix (Section 8.5) against the same heads run one by one
    through the batched call (bit-exact), and layer by layer against the oracle on the head's column block.
    d_h = 50 (bf16) puts the heads off the 16-byte grid: element-wise loader."""
    say("grouped per-head cascade T=%d d=%d H=%d %s" % (T, d, H, dtype))
    w = wl.small(T=T, d=d, K=K, L=L, dtype=dtype, seed=61 + T, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    dh = d // H
    ws = pa.workspace_batched(T, H, DEV)
    grouped = pa.ada_cascade_layers_grouped([pa.heads_view(x, H) for x in xs], w.tau, want_lists=True, ws=ws)
    again = pa.ada_cascade_layers_grouped([pa.heads_view(x, H) for x in xs], w.tau, want_lists=True, ws=ws)
    one_by_one = pa.ada_cascade_layers_batched([[x[:, h * dh:(h + 1) * dh] for x in xs] for h in range(H)], w.tau,
                                               want_lists=True)
    torch.cuda.synchronize()
    counts = grouped["counts"].cpu()
    assert counts[:, :, 3].flatten().tolist() == [0] * (H * L)
    for other in (again, one_by_one):
        assert torch.equal(other["counts"].cpu(), counts) and torch.equal(other["gram_ops"], grouped["gram_ops"])
        for h in range(H):
            for l in range(L):
                r, na, nr = (int(v) for v in counts[h, l, :3])
                assert torch.equal(other["idx"][h, l, :r], grouped["idx"][h, l, :r])
                if l > 0:
                    assert torch.equal(other["adds"][h, l, :na], grouped["adds"][h, l, :na])
                    assert torch.equal(other["removes"][h, l, :nr], grouped["removes"][h, l, :nr])
    idx_all, ops = grouped["idx"].cpu(), grouped["gram_ops"].cpu()
    adds_all, rem_all = grouped["adds"].cpu(), grouped["removes"].cpu()
    for h in range(H if T < 2000 else 2):
        prev = None
        for l in range(L):
            xh = xs_cpu[l][:, h * dh:(h + 1) * dh].contiguous()
            r, na, nr = (int(v) for v in counts[h, l, :3])
            idx = idx_all[h, l, :r].numpy()
            if l == 0:
                ref = oracle.select_full(wl.as_f64(xh), w.tau)
                assert np.array_equal(idx, ref["idx"]) and int(ops[h, 0]) == T * T
            else:
                got = dict(idx=idx, adds=adds_all[h, l, :na].numpy(), removes=rem_all[h, l, :nr].numpy(),
                           gram_ops=int(ops[h, l]), r=r, n_adds=na, n_removes=nr,
                           gamma=pa.fetch(pa.ada_cascade_step(xs[l][:, h * dh:(h + 1) * dh], w.tau, dev_idx(prev)))["gamma"])
                parity.check_cascade(xh, w.tau, prev, got, what="grouped head %d layer %d" % (h, l))
            prev = idx


@pytest.mark.parametrize("flags", [0, pa.FLAG_CROSS_EARLIER_ONLY, pa.FLAG_TWO_PASS])
def test_grouped_step_on_stacked_sequences(flags):
    """ada_cascade_step_grouped on G sequences stacked in one [G, T, d] tensor, with the inherited counts on the host
    (a common bound r) and on the device, against single ada_cascade_step calls and the oracle; one group's list is
    bad and only that group reports it."""
    G, T, d = 5, 450, 256
    say("grouped step, stacked sequences G=%d T=%d d=%d flags=%d" % (G, T, d, flags))
    w = wl.small(T=T, d=d, K=60, L=2, dtype="bf16", seed=71, p=0.15)
    seqs_cpu = [wl.layer_list(w, sequence=b) for b in range(G)]
    x0 = torch.stack([s[0] for s in seqs_cpu]).to(DEV)
    x1 = torch.stack([s[1] for s in seqs_cpu]).to(DEV)
    sel = pa.ada_select_full_grouped(x0, w.tau)                 # layer 0 of all sequences in the same launches
    prev, cnt = sel["idx"], sel["counts"]
    prev_sets = []
    for b in range(G):
        f = pa.fetch(pa.ada_select_full(x0[b], w.tau))
        parity.check_full(seqs_cpu[b][0], w.tau, f, "stacked seq %d" % b)
        r = int(cnt[b, 0])
        assert np.array_equal(prev[b, :r].cpu().numpy(), f["idx"]) and cnt[b].cpu().tolist() == [r, r, 0, 0]
        assert np.array_equal(sel["mask"][b].cpu().numpy(), f["mask"])
        prev_sets.append(np.asarray(f["idx"]))
    out = pa.ada_cascade_step_grouped(x1, w.tau, prev, r=T, r_dev=cnt, flags=flags)
    torch.cuda.synchronize()
    c = out["counts"].cpu()
    assert c[:, 3].tolist() == [0] * G
    for b in range(G):
        r, na, nr = (int(v) for v in c[b, :3])
        single = pa.fetch(pa.ada_cascade_step(x1[b], w.tau, dev_idx(prev_sets[b]), flags=flags))
        got = dict(idx=out["idx"][b, :r].cpu().numpy(), adds=out["adds"][b, :na].cpu().numpy(),
                   removes=out["removes"][b, :nr].cpu().numpy(), gram_ops=int(out["gram_ops"][b]), r=r, n_adds=na,
                   n_removes=nr, gamma=single["gamma"])
        assert np.array_equal(got["idx"], single["idx"]) and got["gram_ops"] == single["gram_ops"]
        parity.check_cascade(seqs_cpu[b][1], w.tau, prev_sets[b], got, flags=oflags(flags), what="grouped seq %d" % b,
                             two_pass=bool(flags & pa.FLAG_TWO_PASS))
    # host-side count: every group inherits the same number of tokens (the first 20 of its set)
    out2 = pa.ada_cascade_step_grouped(x1, w.tau, prev, r=20, flags=flags)
    for b in range(G):
        single = pa.fetch(pa.ada_cascade_step(x1[b], w.tau, dev_idx(prev_sets[b][:20]), flags=flags))
        r = int(out2["counts"][b, 0])
        assert np.array_equal(out2["idx"][b, :r].cpu().numpy(), single["idx"])
    # a list that is not ascending in group 3 only
    bad = prev.clone()
    bad[3, 1] = bad[3, 0]
    out3 = pa.ada_cascade_step_grouped(x1, w.tau, bad, r=T, r_dev=cnt, flags=flags)
    st = out3["counts"][:, 3].cpu().tolist()
    assert st[3] == 4 and [st[b] for b in (0, 1, 2, 4)] == [0, 0, 0, 0]
    assert torch.equal(out3["idx"][0, :int(c[0, 0])], out["idx"][0, :int(c[0, 0])])


def test_layer_loop_replays_from_a_hip_graph():
    """The layer loop enqueues kernels only (flags and counters are cleared by kernels, never by memset nodes), so a
    stream capture of it replays: three replays with eager work and synchronisation in between, each compared with
    the eager result; then new activations are copied into the captured buffers and the replay follows them."""
    say("HIP graph replay of ada_cascade_layers")
    w = wl.small(T=700, d=256, K=90, L=5, dtype="bf16", seed=131, p=0.1)
    xs = [x.to(DEV) for x in wl.layer_list(w)]
    other = [x.to(DEV) for x in wl.layer_list(w, sequence=1)]
    ws = pa.workspace(w.T, DEV)
    out = dict(idx=torch.zeros((w.L, w.T), dtype=torch.int32, device=DEV),
               counts=torch.zeros((w.L, 4), dtype=torch.int32, device=DEV),
               gram_ops=torch.zeros(w.L, dtype=torch.int64, device=DEV))
    eager = run_driver(xs, w.tau, want_lists=False)
    eager_other = run_driver(other, w.tau, want_lists=False)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                # warm-up outside the capture (one-time attribute calls)
        pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out)

    def same(a):
        c = out["counts"].cpu()
        assert torch.equal(c, a["counts"].cpu()) and torch.equal(out["gram_ops"], a["gram_ops"])
        for l in range(w.L):
            assert torch.equal(out["idx"][l, :int(c[l, 0])], a["idx"][l, :int(c[l, 0])])

    for rep in range(3):
        out["counts"].zero_()
        out["idx"].zero_()
        graph.replay()
        torch.cuda.synchronize()
        same(eager)
        run_driver(other, w.tau, want_lists=False)               # eager work of the library between replays
    for x, y in zip(xs, other):
        x.copy_(y)
    graph.replay()
    torch.cuda.synchronize()
    same(eager_other)


@pytest.mark.parametrize("T,H,dh,K,L,dtype", [(600, 4, 64, 70, 4, "bf16"), (333, 2, 64, 40, 3, "f32"), (1500, 3, 128, 200, 3, "bf16")])
def test_selection_pipelined_against_attention(T, H, dh, K, L, dtype):
    """ada_pipeline_layers on two streams and on one: sets, assignment and attention output of every layer equal
    those of the single calls (same kernels: bit-exact), and the attention output is checked against the oracle on
    the set and assignment the layer used."""
    d = H * dh
    say("pipeline T=%d H=%d d_h=%d L=%d %s" % (T, H, dh, L, dtype))
    w = wl.small(T=T, d=d, K=K, L=L, dtype=dtype, seed=151 + T, p=0.1)
    xs_cpu = wl.layer_list(w)
    qkv_cpu = [wl.qkv(w, H, layer=l) for l in range(L)]
    xs = [x.to(DEV) for x in xs_cpu]
    qs, ks, vs = ([t[i].to(DEV) for t in qkv_cpu] for i in range(3))
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    chain = run_driver(xs, w.tau, want_lists=False)
    cc = chain["counts"].cpu()
    for streams in ((s1, s2), (None, None), (s1, s1)):
        res = pa.ada_pipeline_layers(xs, qs, ks, vs, H, w.tau, stream_sel=streams[0], stream_attn=streams[1])
        counts = res["counts"].cpu()                              # on the caller's stream: joined with both
        info = res["info"].cpu()
        assert torch.equal(counts, cc) and torch.equal(res["gram_ops"], chain["gram_ops"])
        assert info[:, 3].tolist() == [0] * L and info[:, 7].tolist() == [0] * L
        for l in range(L):
            r = int(counts[l, 0])
            idx = res["idx"][l, :r]
            assert torch.equal(idx, chain["idx"][l, :r])
            near = pa.ada_assign_nearest(xs[l], idx.contiguous())
            assert torch.equal(near["assign"], res["assign"][l])
            att = pa.ada_attention_compressed(qs[l], ks[l], vs[l], H, idx.contiguous(), near["assign"])
            assert torch.equal(att["out"], res["out"][l])
            assert int(info[l, 0]) == T - r and int(info[l, 4]) == r
    for l in (0, L - 1):
        r = int(counts[l, 0])
        parity.check_attention(qkv_cpu[l][0], qkv_cpu[l][1], qkv_cpu[l][2], H, res["idx"][l, :r].cpu().numpy(),
                               res["assign"][l].cpu().numpy(), res["out"][l].cpu().numpy(), what="pipeline layer %d" % l)


def greedy_reference(x_cpu, tau, got_mask):
    """The oracle's greedy covering with the decisions of band tokens (oracle gamma within the band of the threshold)
    taken from the GPU; repeated until no new band token appears, because a forced decision changes which earlier
    representatives later tokens are compared with."""
    X = wl.as_f64(x_cpu)
    T = X.shape[0]
    force = -np.ones(T, dtype=np.int8)
    for _ in range(8):
        ref = oracle.select_full(X, tau, greedy=True, force=force)
        band = (np.abs(ref["gamma"] - parity.thr_of(tau)) < parity.BAND) & (force < 0)
        if not band.any():
            return ref
        force[band] = got_mask[band]
    raise AssertionError("band tokens keep appearing")


def chain_rows(T, d, seed):
    """Unit vectors in a plane embedded in d dimensions, at angles that form long chains (each token within the
    threshold of its neighbours but not of tokens further away), in shuffled order, plus exact duplicates."""
    rng = np.random.default_rng(seed)
    ang = rng.uniform(0, np.pi, size=T)
    ang[rng.integers(0, T, size=T // 10)] = ang[rng.integers(0, T, size=T // 10)]
    basis = np.linalg.qr(rng.standard_normal((d, 2)))[0]
    X = (np.cos(ang)[:, None] * basis[:, 0] + np.sin(ang)[:, None] * basis[:, 1]) * rng.uniform(0.5, 2.0, size=(T, 1))
    return X


@pytest.mark.parametrize("T,d,dtype", [(1, 64, "bf16"), (64, 32, "f32"), (130, 64, "bf16"), (333, 96, "f32"), (700, 256, "bf16"),
                                       (1290, 128, "bf16"), (2048, 64, "bf16"), (3000, 32, "bf16"), (2060, 64, "bf16"),
                                       (2100, 96, "bf16"), (5000, 32, "bf16")])
def test_greedy_covering_selection(T, d, dtype):
    """ADA_FLAG_GREEDY_COVER against the oracle's greedy variant: on chain-rich inputs (where it differs from the
    Definition in many tokens) and on the clustered workload (where the two coincide); both tile sizes."""
    say("greedy covering T=%d d=%d %s" % (T, d, dtype))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x_chain = torch.from_numpy(chain_rows(T, d, 400 + T)).to(torch.float32).to(tdt)
    w = wl.small(T=T, d=d, K=max(1, T // 8), L=1, dtype=dtype, seed=41 + T)
    ws = pa.workspace(T, DEV)
    n_differ = 0
    for name, x_cpu, tau in (("chains", x_chain, 0.05), ("chains", x_chain, 0.3), ("clusters", wl.layer_list(w)[0], w.tau)):
        # the register-staged tiles of both sizes, and the direct-to-LDS kernel with both ways of cutting the triangle
        # (where the shape allows it; otherwise these switches change nothing)
        for var, tile in (("ADA_TILE", "64"), ("ADA_TILE", "128"), ("ADA_GRAM", "tile"), ("ADA_GRAM", "dma0"), ("ADA_GRAM", "dma1"), ("ADA_GRAM", "dma2")):
            os.environ[var] = tile
            try:
                got = pa.fetch(pa.ada_select_full(x_cpu.to(DEV), tau, ws=ws, flags=pa.FLAG_GREEDY_COVER))
            finally:
                del os.environ[var]
            ref = greedy_reference(x_cpu, tau, got["mask"])
            assert np.array_equal(got["mask"], ref["mask"]), "%s tau=%g %s=%s: mask differs at %s" % (
                name, tau, var, tile, np.nonzero(got["mask"] != ref["mask"])[0][:8])
            assert np.array_equal(got["idx"], ref["idx"]) and got["r"] == len(ref["idx"])
            dfn = oracle.select_full(wl.as_f64(x_cpu), tau)
            assert float(np.max(np.abs(got["gamma"].astype(np.float64) - dfn["gamma"]))) <= parity.GAMMA_TOL
            n_differ += int(np.sum(ref["mask"] != dfn["mask"]))
        # the workspace is left usable by the other calls
        parity.check_full(x_cpu, tau, pa.fetch(pa.ada_select_full(x_cpu.to(DEV), tau, ws=ws)), "after greedy")
    if T >= 130:
        assert n_differ > 0                                       # the chain inputs do separate the two readings


def drifting_chain_layers(T, d, L, seed):
    """Layers whose rows are unit vectors spread over a plane (so that the threshold decides how many neighbours a
    token has) and drift a little from layer to layer."""
    rng = np.random.default_rng(seed)
    ang = rng.uniform(0, np.pi, size=T)
    basis = np.linalg.qr(rng.standard_normal((d, 2)))[0]
    out = []
    for _ in range(L):
        out.append(np.cos(ang)[:, None] * basis[:, 0] + np.sin(ang)[:, None] * basis[:, 1])
        ang = ang + rng.normal(0, 0.02, size=T)
    return out


@pytest.mark.parametrize("kind,T,d,dtype,ctl", [("clusters", 600, 192, "bf16", (0.05, 0.8, 0.02, 0.6)),
                                                ("chains", 500, 64, "f32", (0.1, 1.5, 0.05, 0.4)),
                                                ("chains", 1100, 128, "bf16", (0.1, 1.5, 0.05, 0.4)),
                                                ("chains", 700, 96, "bf16", (0.0, 0.3, 0.02, 0.6))])
def test_threshold_adapted_on_the_device(kind, T, d, dtype, ctl):
    """ada_cascade_layers_adaptive: the tau of every layer equals, bit for bit, the rule applied in float64 to the
    previous step's own counts; every step is checked against the oracle at that tau on the set it consumed; and
    the whole trajectory equals the oracle's own adaptive loop when no decision falls into the band."""
    L = 7
    say("adaptive tau %s T=%d d=%d %s ctl=%s" % (kind, T, d, dtype, ctl))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    if kind == "clusters":
        w = wl.small(T=T, d=d, K=70, L=L, dtype=dtype, seed=171, p=0.15)
        xs_cpu, tau0 = wl.layer_list(w), w.tau
    else:
        xs_cpu = [torch.from_numpy(x).to(torch.float32).to(tdt) for x in drifting_chain_layers(T, d, L, 181 + T)]
        tau0 = 0.2
    xs = [x.to(DEV) for x in xs_cpu]
    kappa, eta_t, tmin, tmax = ctl
    out = pa.ada_cascade_layers_adaptive(xs, tau0, kappa, eta_t, tmin, tmax)
    torch.cuda.synchronize()
    counts, taus, thrs = out["counts"].cpu(), out["tau"].cpu().numpy(), out["thr"].cpu().numpy()
    assert counts[:, 3].tolist() == [0] * L
    t32 = float(np.float32(tau0))
    assert taus[0] == t32 and taus[1] == t32
    prev = None
    for l in range(L):
        r, na, nr = (int(v) for v in counts[l, :3])
        idx = out["idx"][l, :r].cpu().numpy()
        assert thrs[l] == np.float32(1.0 - taus[l] * taus[l])
        if l == 0:
            parity.check_full(xs_cpu[0], taus[0], pa.fetch(pa.ada_select_full(xs[0], tau0)), "adaptive layer 0")
            assert np.array_equal(idx, pa.fetch(pa.ada_select_full(xs[0], tau0))["idx"])
        else:
            if l + 1 < L:
                eta = oracle.metrics.turnover(na, nr, len(prev))
                assert taus[l + 1] == oracle.metrics.adapt_tau(float(taus[l]), eta, kappa, eta_t, tmin, tmax)
            got = dict(idx=idx, adds=out["adds"][l, :na].cpu().numpy(), removes=out["removes"][l, :nr].cpu().numpy(),
                       gram_ops=int(out["gram_ops"][l]), r=r, n_adds=na, n_removes=nr,
                       gamma=pa.fetch(pa.ada_cascade_step(xs[l], float(taus[l]), dev_idx(prev)))["gamma"])
            parity.check_cascade(xs_cpu[l], float(taus[l]), prev, got, what="adaptive layer %d tau %.4f" % (l, taus[l]))
        prev = idx
    if kappa != 0.0:
        assert len(set(taus.tolist())) > 2                       # the threshold moved
    if kind == "chains":
        sizes = [int(c) for c in counts[:, 0]]
        fixed = run_driver(xs, tau0, want_lists=False)["counts"][:, 0].cpu().tolist()
        assert (sizes != fixed) == (kappa != 0.0)                # ... and moving it changes the sets on these inputs
    ref_taus, ref = oracle.cascade_layers_adaptive([wl.as_f64(x) for x in xs_cpu], tau0, kappa, eta_t, tmin, tmax)
    if all(np.array_equal(ref[l]["idx"], out["idx"][l, :int(counts[l, 0])].cpu().numpy()) for l in range(L)):
        assert ref_taus == taus.tolist()
    else:                                                          # only a band decision may separate the two loops
        l = next(l for l in range(L) if not np.array_equal(ref[l]["idx"], out["idx"][l, :int(counts[l, 0])].cpu().numpy()))
        g = ref[l]["gamma"]
        assert np.any(np.abs(g - parity.thr_of(ref_taus[l])) < parity.BAND), "loops differ at layer %d without a band token" % l


@pytest.mark.parametrize("T,d,K,dtype", [(4100, 64, 300, "bf16"), (5001, 96, 500, "bf16"), (6000, 32, 900, "f32"), (8192, 128, 400, "bf16"),
                                         (12000, 64, 2500, "bf16")])
def test_cascade_step_on_long_sequences(T, d, K, dtype):
    """Sequences longer than 4096 tokens (odd T: scalar loads in the set update; r above 1024: more than one pass over
    the list): against the oracle, twice on one workspace, with the set size on the host and on the device, for a
    bad list, and with three stacked sequences in one launch."""
    say("long sequence T=%d d=%d K=%d %s" % (T, d, K, dtype))
    w = wl.small(T=T, d=d, K=K, L=3, dtype=dtype, seed=211 + T, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    ws = pa.workspace(T, DEV)
    full = pa.fetch(pa.ada_select_full(xs[0], w.tau, ws=ws))
    prev = full["idx"]
    for l in (1, 2):
        for flags in (0, pa.FLAG_CROSS_EARLIER_ONLY):
            got = pa.fetch(pa.ada_cascade_step(xs[l], w.tau, dev_idx(prev), ws=ws, flags=flags))
            parity.check_cascade(xs_cpu[l], w.tau, prev, got, flags=oflags(flags), what="long sequence layer %d" % l)
        again = pa.fetch(pa.ada_cascade_step(xs[l], w.tau, dev_idx(prev), ws=ws, flags=flags))
        for k in ("idx", "adds", "removes"):
            assert np.array_equal(again[k], got[k])
        # the count on the device, the list padded to T entries
        padded = torch.zeros(T, dtype=torch.int32, device=DEV)
        padded[:len(prev)] = dev_idx(prev)
        cnt = torch.tensor([len(prev), 0, 0, 0], dtype=torch.int32, device=DEV)
        dv = pa.fetch(pa.ada_cascade_step(xs[l], w.tau, padded, r=T, r_dev=cnt, ws=ws, flags=flags))
        for k in ("idx", "adds", "removes"):
            assert np.array_equal(dv[k], got[k])
        prev = pa.fetch(pa.ada_cascade_step(xs[l], w.tau, dev_idx(prev), ws=ws))["idx"]
    bad = np.array(full["idx"], copy=True)
    bad[3] = bad[2]
    res = pa.ada_cascade_step(xs[1], w.tau, dev_idx(bad), ws=ws)
    assert res["counts"].cpu().tolist() == [0, 0, 0, 4]
    parity.check_cascade(xs_cpu[1], w.tau, full["idx"], pa.fetch(pa.ada_cascade_step(xs[1], w.tau, dev_idx(full["idx"]), ws=ws)),
                         what="after a rejected list")
    if T <= 6000:
        G = 3
        seqs_cpu = [wl.layer_list(w, sequence=b, n_layers=2) for b in range(G)]
        xg = [torch.stack([seqs_cpu[b][l] for b in range(G)]).to(DEV) for l in range(2)]
        out = pa.ada_cascade_layers_grouped(xg, w.tau, want_lists=True)
        c = out["counts"].cpu()
        assert c[:, :, 3].flatten().tolist() == [0] * (2 * G)
        for b in range(G):
            single = run_driver([xg[l][b] for l in range(2)], w.tau)
            assert torch.equal(single["counts"].cpu(), c[b])
            r, na, nr = (int(v) for v in c[b, 1, :3])
            assert torch.equal(single["idx"][1, :r], out["idx"][b, 1, :r])
            assert torch.equal(single["adds"][1, :na], out["adds"][b, 1, :na])
            assert torch.equal(single["removes"][1, :nr], out["removes"][b, 1, :nr])


def run_driver(xs, tau, **kw):
    out = pa.ada_cascade_layers(xs, tau, **kw)
    torch.cuda.synchronize()
    return out


def assert_same_driver_output(a, b, L):
    ca, cb = a["counts"].cpu(), b["counts"].cpu()
    assert torch.equal(ca, cb) and torch.equal(a["gram_ops"], b["gram_ops"])
    for l in range(L):
        r, na, nr = (int(v) for v in ca[l, :3])
        assert torch.equal(a["idx"][l, :r], b["idx"][l, :r])
        if l > 0:
            assert torch.equal(a["adds"][l, :na], b["adds"][l, :na])
            assert torch.equal(a["removes"][l, :nr], b["removes"][l, :nr])


@pytest.mark.parametrize("T,d,K,L,dtype", [(600, 192, 70, 6, "bf16"), (333, 96, 40, 5, "f32"), (130, 64, 20, 70, "bf16")])
def test_resident_pass_matches_one_launch_per_layer_and_the_oracle(T, d, K, L, dtype, monkeypatch):
    """The layer loop in one resident launch (rows in whole 128-byte chunks) against the same loop as one launch per
    layer, and layer by layer against the oracle; L = 70 takes two resident launches."""
    say("resident pass T=%d d=%d L=%d %s" % (T, d, L, dtype))
    w = wl.small(T=T, d=d, K=K, L=L, dtype=dtype, seed=17 + L, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    ws = pa.workspace(T, DEV)
    resident = run_driver(xs, w.tau, ws=ws, flags=pa.FLAG_RESIDENT_PASS)
    again = run_driver(xs, w.tau, ws=ws, flags=pa.FLAG_RESIDENT_PASS)    # the workspace is left ready
    chained = run_driver(xs, w.tau, ws=ws)
    assert resident["counts"][:, 3].cpu().tolist() == [0] * L
    assert_same_driver_output(resident, chained, L)
    assert_same_driver_output(resident, again, L)
    counts = resident["counts"].cpu()
    prev = resident["idx"][0, :int(counts[0, 0])].cpu().numpy()
    for l in range(1, min(L, 8)):
        r, na, nr = (int(v) for v in counts[l, :3])
        got = dict(idx=resident["idx"][l, :r].cpu().numpy(), adds=resident["adds"][l, :na].cpu().numpy(),
                   removes=resident["removes"][l, :nr].cpu().numpy(), gram_ops=int(resident["gram_ops"][l]),
                   r=r, n_adds=na, n_removes=nr,
                   gamma=pa.fetch(pa.ada_cascade_step(xs[l], w.tau, dev_idx(prev)))["gamma"])
        parity.check_cascade(xs_cpu[l], w.tau, prev, got, what="resident layer %d" % l)
        prev = got["idx"]


def test_resident_pass_gives_up_cleanly_when_its_wait_is_cut_short(monkeypatch):
    """The wait between layers is bounded.  With the bound forced to a single poll most workgroups give up at the
    second layer: every kernel still ends, unfinished layers report ADA_ERR_DEVICE, finished ones are correct, and a
    re-initialised workspace serves the next call."""
    say("resident pass, spin limit 1")
    w = wl.small(T=700, d=128, K=60, L=5, dtype="bf16", seed=19, p=0.1)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    ws = pa.workspace(w.T, DEV)
    good = run_driver(xs, w.tau, ws=ws)
    monkeypatch.setenv("ADA_SPIN_LIMIT", "1")
    cut = run_driver(xs, w.tau, ws=ws, flags=pa.FLAG_RESIDENT_PASS)
    status = cut["counts"][:, 3].cpu().tolist()
    assert status[0] == 0 and status[1] == 0 and set(status) <= {0, 6}
    done = [l for l in range(w.L) if status[l] == 0]
    assert done == list(range(len(done)))                         # a layer cannot finish after one that did not
    for l in done:
        r = int(cut["counts"][l, 0])
        assert torch.equal(cut["counts"][l], good["counts"][l]) and torch.equal(cut["idx"][l, :r], good["idx"][l, :r])
    monkeypatch.delenv("ADA_SPIN_LIMIT")
    pa.ada_workspace_init(ws)
    assert_same_driver_output(run_driver(xs, w.tau, ws=ws, flags=pa.FLAG_RESIDENT_PASS), good, w.L)


def test_set_overlap():
    say("ada_set_overlap")
    rng = np.random.default_rng(5)
    for T in (1, 77, 5000):
        a = (rng.random(T) < 0.4).astype(np.uint8)
        b = (rng.random(T) < 0.5).astype(np.uint8)
        out = pa.ada_set_overlap(torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)).cpu().tolist()
        assert out == [int((a & b).sum()), int((a | b).sum())]
        A, B = np.flatnonzero(a), np.flatnonzero(b)
        if out[1]:
            assert out[0] / out[1] == pytest.approx(oracle.metrics.jaccard(A, B))


def test_deterministic_reruns():
    say("determinism")
    w = wl.small(T=900, d=256, K=90, L=2, dtype="bf16", seed=91, p=0.1)
    xs = [x.to(DEV) for x in wl.layer_list(w)]
    a = pa.ada_select_full(xs[0], w.tau)
    b = pa.ada_select_full(xs[0], w.tau)
    assert torch.equal(a["gamma"], b["gamma"]) and torch.equal(a["mask"], b["mask"])   # max is order-independent
    c = pa.ada_cascade_step(xs[1], w.tau, a["idx"], r=w.T, r_dev=a["counts"])
    d = pa.ada_cascade_step(xs[1], w.tau, a["idx"], r=w.T, r_dev=a["counts"])
    assert torch.equal(c["gamma"], d["gamma"]) and torch.equal(c["counts"], d["counts"])


@pytest.mark.parametrize("ci,groups", [(2, 1), (3, 1), (2, 4)])
def test_repeated_passes_are_bit_identical(ci, groups):
    """300 passes of the layer loop at the benchmark's shapes (one sequence of configurations 2 and 3; four stacked
    sequences of configuration 2 in one launch per step): every pass must reproduce pass 0 bit for bit (index sets,
    counts, Gram-operation counts).  The hand-over between workgroups inside a launch (hit words and first-hit records
    written through the L2, tickets, one cache invalidate) and the workspace's zero-between-calls state are what this
    exercises; pass 0 itself is the one the configuration tests check against the oracle."""
    w = wl.config(ci)
    n_layers = 10
    say("%s: 300 passes, %d layers, %d group(s)" % (w.name, n_layers, groups))
    if groups == 1:
        xs = [x.to(DEV) for x in wl.layers(w, 0, n_layers)]
        ws = pa.workspace(w.T, DEV)
        run = lambda out: pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out, want_lists=True)
    else:
        per = [wl.layer_list(w, b, n_layers) for b in range(groups)]
        xg = [torch.stack([per[b][l] for b in range(groups)]).to(DEV) for l in range(n_layers)]
        ws = pa.workspace_batched(w.T, groups, DEV)
        run = lambda out: pa.ada_cascade_layers_grouped(xg, w.tau, ws=ws, out=out, want_lists=True)
    out = run(None)
    torch.cuda.synchronize()
    keys = ("idx", "counts", "gram_ops", "adds", "removes")
    for k in keys:                                   # unwritten tails must compare equal too: start them from zero
        out[k].zero_()
    out = run(out)
    torch.cuda.synchronize()
    first = {k: out[k].clone() for k in keys}
    assert first["counts"].reshape(-1, 4)[:, 3].abs().sum().item() == 0
    for i in range(1, 300):
        out = run(out)
        for k in keys:
            assert torch.equal(out[k], first[k]), "pass %d differs from pass 0 in %s" % (i, k)


# ------------------------------------------------------------------------------------------ the five configurations
def test_config0_all_layers():
    w = wl.config(0)
    say(w.name)
    stats = run_layers_teacher_forced(w, wl.layer_list(w), what=w.name)
    assert sum(a + r for a, r, _ in stats) > 0


def test_config1_all_layers_with_full_selection_at_every_layer():
    w = wl.config(1)
    say(w.name)
    xs_cpu = wl.layer_list(w)
    run_layers_teacher_forced(w, xs_cpu, what=w.name)
    for l in range(w.L):                      # the configuration's comparison path: the full selection at every layer
        parity.check_full(xs_cpu[l], w.tau, pa.fetch(pa.ada_select_full(xs_cpu[l].to(DEV), w.tau)),
                          "%s full layer %d" % (w.name, l))


CUS = 256     # workgroups that share a single problem's tiles on this device (what ada_plan_tile_shape is asked with)


@pytest.mark.parametrize("ci,full_every", [(2, 1), (3, 4)])
def test_config2_and_3_all_layers(ci, full_every):
    """Every layer of the configuration, teacher-forced: the cascade set grows and shrinks with depth, so the later
    layers reach representative-block counts (and with them tile plans and set-update forms) that the first few do
    not.  The full selection (the configuration's comparison path) is checked at every `full_every`-th layer."""
    w = wl.config(ci)
    say("%s, all %d layers" % (w.name, w.L))
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    assert pa.ada_plan_full_units(w.T, w.d, CUS) == 2            # T = 2048: 64 x 128 units and the diagonal units, one launch
    full = pa.fetch(pa.ada_select_full(xs[0], w.tau))
    parity.check_full(xs_cpu[0], w.tau, full, w.name + " layer 0")
    prev = full["idx"]
    inherited, moved = [], 0
    for l in range(1, w.L):
        say("%s layer %d, r=%d" % (w.name, l, len(prev)))
        inherited.append(len(prev))
        got, _ = step_and_check(xs[l], xs_cpu[l], w.tau, prev, 0, "%s layer %d" % (w.name, l))
        moved += got["n_adds"] + got["n_removes"]
        prev = got["idx"]
        if l % full_every == 0:
            parity.check_full(xs_cpu[l], w.tau, pa.fetch(pa.ada_select_full(xs[l], w.tau)), "%s full layer %d" % (w.name, l))
    assert moved > 0
    shapes = {pa.ada_plan_tile_shape(r, w.T, w.d, CUS) for r in inherited}
    say("%s: inherited sizes %d..%d, tile plans %s" % (w.name, min(inherited), max(inherited), sorted(shapes)))
    assert shapes == {EXPECTED_PLANS[ci]}, shapes
    blocks64 = {(r + 63) // 64 for r in inherited}
    if ci == 2:
        assert len(blocks64) > 1, "the set never crossed a 64-representative block boundary"
        assert max(inherited) <= 512 and min(inherited) > 384     # one update form, both sides of 448
    else:
        assert min(inherited) > 512 and max(inherited) <= 1024    # the 32-word update form


# the tile plan (ada_plan_tile_shape) each configuration's single-sequence cascade step is meant to take
EXPECTED_PLANS = {2: 0, 3: 1, 4: 3}


@pytest.fixture(scope="module")
def config4_batch():
    """The long-sequence configuration as it is stated: four sequences with their own seeds, stacked in one tensor per
    layer, layers 0..8 (the full selection at layer 0, eight cascade steps; layer 8 is where the configuration asks for
    the next full selection).  One stacked GPU pass; the tests below check every sequence against the oracle."""
    w = wl.config(4)
    n_layers = 9
    say("%s: generating %d sequences x %d layers" % (w.name, w.batch, n_layers))
    seqs_cpu = [wl.layer_list(w, b, n_layers) for b in range(w.batch)]
    xg = [torch.stack([seqs_cpu[b][l] for b in range(w.batch)]).to(DEV) for l in range(n_layers)]
    out = pa.ada_cascade_layers_grouped(xg, w.tau, want_lists=True)
    torch.cuda.synchronize()
    host = {k: v.cpu() for k, v in out.items() if isinstance(v, torch.Tensor)}
    return w, n_layers, seqs_cpu, xg, host


def full_selection_sampled(X64, tau, idx, rows, what):
    ref = oracle.gamma_full_rows(X64, rows)
    assert np.all(np.abs(ref - parity.thr_of(tau)) > parity.BAND), what
    assert np.array_equal(np.isin(rows, idx), ref < parity.thr_of(tau)), what


@pytest.mark.parametrize("b", [0, 1, 2, 3])
def test_config4_every_sequence_of_the_stacked_batch(config4_batch, b):
    """Sequence b of the stacked pass: every cascade step against the oracle (teacher-forced), the layer-0 selection
    completely for sequence 0 and on sampled tokens for the others."""
    w, n_layers, seqs_cpu, xg, out = config4_batch
    counts = out["counts"]
    assert counts[:, :, 3].flatten().tolist() == [0] * (w.batch * n_layers)
    assert len({tuple(counts[s, :, 0].tolist()) for s in range(w.batch)}) == w.batch          # the sequences differ
    rng = np.random.default_rng(40 + b)
    prev = None
    single_plans, stacked_plans = set(), set()
    for l in range(n_layers):
        r, na, nr = (int(v) for v in counts[b, l, :3])
        idx = out["idx"][b, l, :r].numpy()
        say("%s sequence %d layer %d, r=%d" % (w.name, b, l, r))
        if l == 0:
            X0 = wl.as_f64(seqs_cpu[b][0])
            if b == 0:
                ref = oracle.select_full(X0, w.tau)
                assert np.all(np.abs(ref["gamma"] - parity.thr_of(w.tau)) > parity.BAND)
                assert np.array_equal(idx, ref["idx"])
            else:
                rows = np.unique(np.concatenate([[0, 1, 255, 256, w.T - 1], rng.integers(0, w.T, 40)]))
                full_selection_sampled(X0, w.tau, idx, rows, "%s sequence %d layer 0" % (w.name, b))
        else:
            single_plans.add(pa.ada_plan_tile_shape(len(prev), w.T, w.d, CUS))
            stacked_plans.add(pa.ada_plan_tile_shape(len(prev), w.T, w.d, CUS // w.batch))
            got = dict(idx=idx, adds=out["adds"][b, l, :na].numpy(), removes=out["removes"][b, l, :nr].numpy(),
                       gram_ops=int(out["gram_ops"][b, l]), r=r, n_adds=na, n_removes=nr,
                       gamma=pa.fetch(pa.ada_cascade_step(xg[l][b], w.tau, dev_idx(prev)))["gamma"])
            parity.check_cascade(seqs_cpu[b][l], w.tau, prev, got, what="%s seq %d layer %d" % (w.name, b, l))
        prev = idx
    say("%s sequence %d: tile plans single %s, stacked %s" % (w.name, b, sorted(single_plans), sorted(stacked_plans)))
    # (the first step inherits about 400 representatives, four blocks of 128: one round of 128 x 128 tiles; the set then
    # grows past 512 and the steps take the 128 x 256 tile)
    assert EXPECTED_PLANS[4] in single_plans and single_plans <= {2, EXPECTED_PLANS[4]}, single_plans


@pytest.mark.parametrize("layer", [0, 8])
def test_config4_full_selection_compared_completely(config4_batch, layer):
    """T = 8192, d = 4096 in the launch configuration the benchmark times: mask, index list and every gamma_t against
    the oracle, at layer 0 and at layer 8 (the layers at which the configuration runs the full selection)."""
    w, n_layers, seqs_cpu, xg, _ = config4_batch
    say("%s sequence 0 layer %d: complete full selection" % (w.name, layer))
    assert pa.ada_plan_full_units(w.T, w.d, CUS) == 1            # 256 x 256 units and the unit queue
    got = pa.fetch(pa.ada_select_full(xg[layer][0], w.tau))
    info = parity.check_full(seqs_cpu[0][layer], w.tau, got, "%s full layer %d" % (w.name, layer))
    say("gamma error %.3g, %d tokens in the band" % (info["gamma_err"], info["n_band"]))
    assert got["mask"][0] == 1 and got["r"] == int(got["mask"].sum())


def test_config4_single_sequence_step_in_both_forms(config4_batch):
    """One sequence on its own (the single-problem launch configuration): a deep cascade step in the one-launch and
    the two-launch form, the latter returning Algorithm 1's gamma^cross itself."""
    w, n_layers, seqs_cpu, xg, out = config4_batch
    b, l = 1, 6
    r = int(out["counts"][b, l - 1, 0])
    prev = out["idx"][b, l - 1, :r].numpy()
    for flags in (0, pa.FLAG_TWO_PASS):
        step_and_check(xg[l][b], seqs_cpu[b][l], w.tau, prev, flags, "%s seq %d layer %d flags %d" % (w.name, b, l, flags))


@pytest.mark.parametrize("ci,B,n_layers,checked", [(2, 4, 4, (0, 1, 2, 3))])
def test_stacked_batch_at_full_size(ci, B, n_layers, checked):
    """The batch of the long-context configuration (four sequences with different seeds) and of the benchmark's
    configuration, stacked in one tensor per layer as bench.py runs them: one launch per step for all sequences.
    Every sequence equals its own single-sequence run bit for bit; the sequences in `checked` are also checked
    step by step against the oracle (their full selection on sampled gamma_t at T = 8192)."""
    w = wl.config(ci)
    say("%s: %d stacked sequences, %d layers" % (w.name, B, n_layers))
    seqs_cpu = [wl.layer_list(w, b, n_layers) for b in range(B)]
    xg = [torch.stack([seqs_cpu[b][l] for b in range(B)]).to(DEV) for l in range(n_layers)]
    out = pa.ada_cascade_layers_grouped(xg, w.tau, want_lists=True)
    torch.cuda.synchronize()
    counts = out["counts"].cpu()
    assert counts[:, :, 3].flatten().tolist() == [0] * (B * n_layers)
    for b in range(B):
        single = run_driver([xg[l][b] for l in range(n_layers)], w.tau)
        assert torch.equal(single["counts"].cpu(), counts[b]) and torch.equal(single["gram_ops"], out["gram_ops"][b])
        for l in range(n_layers):
            r, na, nr = (int(v) for v in counts[b, l, :3])
            assert torch.equal(single["idx"][l, :r], out["idx"][b, l, :r])
            if l > 0:
                assert torch.equal(single["adds"][l, :na], out["adds"][b, l, :na])
                assert torch.equal(single["removes"][l, :nr], out["removes"][b, l, :nr])
    assert len({tuple(counts[b, :, 0].tolist()) for b in range(B)}) > 1          # the sequences differ
    rng = np.random.default_rng(ci)
    for b in checked:
        prev = None
        for l in range(n_layers):
            r, na, nr = (int(v) for v in counts[b, l, :3])
            idx = out["idx"][b, l, :r].cpu().numpy()
            if l == 0:
                X0 = wl.as_f64(seqs_cpu[b][0])
                if w.T <= 2048:
                    assert np.array_equal(idx, oracle.select_full(X0, w.tau)["idx"])
                else:
                    rows = np.unique(np.concatenate([[0, 1, w.T - 1], rng.integers(0, w.T, 40)]))
                    ref = oracle.gamma_full_rows(X0, rows)
                    assert np.all(np.abs(ref - parity.thr_of(w.tau)) > parity.BAND)
                    member = np.isin(rows, idx)
                    assert np.array_equal(member, ref < parity.thr_of(w.tau))
            else:
                got = dict(idx=idx, adds=out["adds"][b, l, :na].cpu().numpy(), removes=out["removes"][b, l, :nr].cpu().numpy(),
                           gram_ops=int(out["gram_ops"][b, l]), r=r, n_adds=na, n_removes=nr,
                           gamma=pa.fetch(pa.ada_cascade_step(xg[l][b], w.tau, dev_idx(prev)))["gamma"])
                parity.check_cascade(seqs_cpu[b][l], w.tau, prev, got, what="%s seq %d layer %d" % (w.name, b, l))
            prev = idx


# ------------------------------------------------------------------------------------------ Section 2.3: assignment
def assign_and_check(x_cpu, idx, what, **kw):
    res = pa.ada_assign_nearest(x_cpu.to(DEV), torch.as_tensor(np.asarray(idx, dtype=np.int32)).to(DEV), **kw)
    info = res["info"].cpu().tolist()
    assert info[3] == 0 and info[0] == x_cpu.shape[0] - len(idx), what
    return parity.check_assign(x_cpu, idx, res["assign"].cpu().numpy(), res["corr"].cpu().numpy(), what)


def test_beyond_the_one_launch_limit():
    """T = 16500 > 16384: the cascade step takes its two-launch form whatever the flags say (exact gamma^cross), the
    full selection runs on 256 x 256 units, the assignment on the tile engine without a hit table."""
    w = wl.small(T=16500, d=64, K=300, L=2, dtype="bf16", seed=12, p=0.05)
    say("T=%d beyond the one-launch limit" % w.T)
    xs_cpu = wl.layer_list(w)
    xs = [x.to(DEV) for x in xs_cpu]
    full = pa.fetch(pa.ada_select_full(xs[0], w.tau))
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 16383, 16384, 16499], rng.integers(0, w.T, 200)]))
    ref = oracle.gamma_full_rows(wl.as_f64(xs_cpu[0]), rows)
    assert np.max(np.abs(full["gamma"][rows] - ref)) <= parity.GAMMA_TOL
    clear = np.abs(ref - parity.thr_of(w.tau)) > parity.BAND
    assert np.array_equal(full["mask"][rows][clear], (ref < parity.thr_of(w.tau)).astype(np.uint8)[clear])
    assert full["mask"][0] == 1 and np.array_equal(full["idx"], np.flatnonzero(full["mask"]))
    got = pa.fetch(pa.ada_cascade_step(xs[1], w.tau, dev_idx(full["idx"])))
    parity.check_cascade(xs_cpu[1], w.tau, full["idx"], got, what="T=16500 step", two_pass=True)
    assign_and_check(xs_cpu[1], got["idx"], "T=16500 assign")


@pytest.mark.parametrize("T,d,K,dtype", [(333, 200, 40, "bf16"), (700, 4096, 120, "bf16"), (513, 768, 100, "f32"),
                                         (1000, 64, 90, "bf16"), (129, 33, 8, "f32"), (1, 64, 1, "bf16")])
def test_assignment_small_shapes(T, d, K, dtype):
    """Nearest representatives of the full selection's set and of a cascade step's set, on ragged shapes that take
    the direct-to-LDS and the register-staged loaders."""
    say("assign T=%d d=%d %s" % (T, d, dtype))
    w = wl.small(T=T, d=d, K=K, L=2, dtype=dtype, seed=61 + T, p=0.1)
    xs = wl.layer_list(w)
    full = pa.fetch(pa.ada_select_full(xs[0].to(DEV), w.tau))
    assign_and_check(xs[0], full["idx"], "assign after full T=%d" % T)
    step = pa.fetch(pa.ada_cascade_step(xs[1].to(DEV), w.tau, torch.as_tensor(full["idx"]).to(DEV)))
    assign_and_check(xs[1], step["idx"], "assign after cascade T=%d" % T)


@pytest.mark.parametrize("kgroups", ["1", "2"])
def test_assignment_forms_and_device_count(kgroups, monkeypatch):
    monkeypatch.setenv("ADA_KGROUPS", kgroups)
    say("assign forms kgroups=%s" % kgroups)
    w = wl.small(T=600, d=256, K=70, L=1, dtype="bf16", seed=7, p=0.1)
    x = wl.layer_list(w)[0]
    out = pa.ada_select_full(x.to(DEV), w.tau)
    full = pa.fetch(out)
    # chained on the device: idx buffer of capacity T, size taken from the selection's count
    res = pa.ada_assign_nearest(x.to(DEV), out["idx"], r=w.T, r_dev=out["counts"])
    assert res["info"].cpu().tolist() == [w.T - full["r"], 0, 0, 0]
    parity.check_assign(x, full["idx"], res["assign"].cpu().numpy(), res["corr"].cpu().numpy(), "r_dev")


def test_assignment_extremes_signs_and_ties():
    say("assign extremes")
    rng = np.random.default_rng(5)
    X = torch.tensor(rng.standard_normal((96, 48)), dtype=torch.float32)
    X[40] = -X[3]                      # |G| = 1 with an earlier member, opposite sign
    X[10] = X[80]                      # duplicate of a LATER member of R
    X[50] = 0.0                        # zero row: every cosine 0 -> smallest member of R
    R = [3, 7, 80, 90]
    got = assign_and_check(X, R, "extremes")
    a = pa.ada_assign_nearest(X.to(DEV), torch.tensor(R, dtype=torch.int32, device=DEV))["assign"].cpu().tolist()
    assert a[40] == 3 and a[10] == 80 and a[50] == 3 and got["n_differ"] == 0
    assign_and_check(X, [0], "single representative")
    assign_and_check(X, list(range(96)), "everybody is a representative")


def test_assignment_rejects_bad_sets_on_the_device_and_leaves_the_workspace_clean():
    say("assign bad sets")
    w = wl.small(T=200, d=64, K=20, L=1, dtype="bf16", seed=3)
    x = wl.layer_list(w)[0]
    xd = x.to(DEV)
    ws = pa.workspace(w.T, DEV)
    for bad in ([5, 4, 9], [0, 0, 1], [0, 300], [-1, 2]):
        res = pa.ada_assign_nearest(xd, torch.tensor(bad, dtype=torch.int32, device=DEV), ws=ws)
        assert res["info"].cpu().tolist()[3] == 4, bad            # ADA_ERR_INDEX
    zero = torch.zeros(1, dtype=torch.int32, device=DEV)
    res = pa.ada_assign_nearest(xd, torch.tensor([1, 2, 3], dtype=torch.int32, device=DEV), r_dev=zero, ws=ws)
    assert res["info"].cpu().tolist()[3] == 2                     # ADA_ERR_SHAPE
    full = pa.fetch(pa.ada_select_full(xd, w.tau, ws=ws))        # the same workspace still serves every call
    parity.check_full(x, w.tau, full, "after bad sets")
    res = pa.ada_assign_nearest(xd, torch.as_tensor(full["idx"]).to(DEV), ws=ws)
    parity.check_assign(x, full["idx"], res["assign"].cpu().numpy(), res["corr"].cpu().numpy(), "after bad sets")


def test_assignment_at_config2_size():
    say("assign config 2")
    w = wl.config(2)
    x = next(iter(wl.layers(w, 0, 1)))
    full = pa.fetch(pa.ada_select_full(x.to(DEV), w.tau))
    got = assign_and_check(x, full["idx"], "config 2")
    assert got["n_differ"] == 0                                   # clusters: the maximiser is unique by a wide margin


# ------------------------------------------------------------------------------------------ eq. (1): attention on R
# Tolerance: products of bf16 (or fp32) inputs are exact in the fp32 accumulators; a score sums d_h <= 256 of them
# (relative rounding ~ d_h 2^-24 of a value of size ~ sqrt(d_h) before scaling: < 1e-5 absolute on scores of order
# 1), exp and the running rescale add a few ulp, bf16 weights are split into hi + lo (2^-17 relative), and the second
# product sums r <= 1000 non-negative weights (sum 1) times values in fp32 (~ 1e-6 |V|).  Measured: up to 6e-6 at
# |V|max = 4.5; the bar is 2e-5 |V|max.
def attention_case(T, d, H, K, dtype, seed, causal, what):
    w = wl.small(T=T, d=d, K=K, L=1, dtype=dtype, seed=seed, p=0.1)
    x = wl.layer_list(w)[0]
    q, k, v = wl.qkv(w, H)
    full = pa.fetch(pa.ada_select_full(x.to(DEV), w.tau))
    idx = torch.as_tensor(full["idx"]).to(DEV)
    near = pa.ada_assign_nearest(x.to(DEV), idx)
    res = pa.ada_attention_compressed(q.to(DEV), k.to(DEV), v.to(DEV), H, idx, near["assign"],
                                      flags=pa.FLAG_ATTN_CAUSAL if causal else 0)
    info = res["info"].cpu().tolist()
    assert info == [full["r"], 0, 0, 0], what
    return parity.check_attention(q, k, v, H, full["idx"], near["assign"].cpu().numpy(), res["out"].cpu().numpy(),
                                  causal, what)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("T,d,H,K,dtype", [(333, 256, 4, 40, "bf16"), (700, 256, 2, 150, "bf16"), (500, 512, 2, 90, "bf16"),
                                           (300, 128, 2, 70, "f32"), (260, 256, 2, 33, "f32"), (1, 64, 1, 1, "bf16"),
                                           (130, 128, 1, 130, "bf16")])
def test_attention_on_the_representative_set(T, d, H, K, dtype, causal):
    """Head sizes 64 / 128 / 256 (bf16) and 64 / 128 (fp32), one to three key blocks, a single token, r = T."""
    say("attention T=%d d=%d H=%d %s causal=%s" % (T, d, H, dtype, causal))
    attention_case(T, d, H, K, dtype, 5 + T, causal, "attention T=%d" % T)


def test_attention_with_device_side_set_size_loops_over_query_blocks():
    """128 heads and the set size on the device: the grid is sized for the chip (two workgroups per head) and each
    workgroup walks through two of the four query blocks."""
    say("attention r_dev, looping grid")
    w = wl.small(T=300, d=8192, K=1000, L=1, dtype="bf16", seed=77, p=0.1)
    x = wl.layer_list(w)[0]
    q, k, v = wl.qkv(w, 128)
    sel = pa.ada_select_full(x.to(DEV), w.tau)
    full = pa.fetch(sel)
    assert full["r"] > 192
    near = pa.ada_assign_nearest(x.to(DEV), sel["idx"], r=w.T, r_dev=sel["counts"])
    res = pa.ada_attention_compressed(q.to(DEV), k.to(DEV), v.to(DEV), 128, sel["idx"], near["assign"], r=w.T,
                                      r_dev=sel["counts"])
    assert res["info"].cpu().tolist() == [full["r"], 0, 0, 0]
    parity.check_attention(q, k, v, 128, full["idx"], near["assign"].cpu().numpy(), res["out"].cpu().numpy(), False,
                           "looping grid")


@pytest.mark.parametrize("causal", [False, True])
def test_attention_long_sequence_hands_over_in_chunks(causal):
    """T = 4500: the hand-over reads the tokens' positions 2048 at a time (three rounds), five key blocks."""
    say("attention T=4500 causal=%s" % causal)
    attention_case(4500, 256, 2, 300, "bf16", 91, causal, "attention T=4500")


def test_attention_one_representative_owns_every_token():
    """One cluster, T = 3000: |R| = 1, so one workgroup per head hands its single row to all 3000 tokens (full lists of
    2048 takers, then 952), and the wave that owns the upper key half never sees a valid key."""
    say("attention, one representative for 3000 tokens")
    w = wl.small(T=3000, d=256, K=1, L=1, dtype="bf16", seed=8, p=0.0)
    x = wl.layer_list(w)[0]
    q, k, v = wl.qkv(w, 2)
    full = pa.fetch(pa.ada_select_full(x.to(DEV), w.tau))
    assert full["r"] == 1
    idx = torch.as_tensor(full["idx"]).to(DEV)
    near = pa.ada_assign_nearest(x.to(DEV), idx)
    for causal in (False, True):
        res = pa.ada_attention_compressed(q.to(DEV), k.to(DEV), v.to(DEV), 2, idx, near["assign"],
                                          flags=pa.FLAG_ATTN_CAUSAL if causal else 0)
        assert res["info"].cpu().tolist() == [1, 0, 0, 0]
        out = res["out"].cpu().numpy()
        parity.check_attention(q, k, v, 2, full["idx"], near["assign"].cpu().numpy(), out, causal, "one representative")
        assert np.array_equal(out, np.broadcast_to(out[0], out.shape))      # every token holds the same row, bit for bit
        # softmax over one key: the row is that key's value row exactly
        assert np.array_equal(out[0], wl.as_f64(v)[int(full["idx"][0])].astype(np.float32))


@pytest.mark.parametrize("gain", [16.0, 64.0])
def test_attention_with_steep_scores_moves_the_reference(gain):
    """Queries scaled by a power of two (exact in bf16): scores spread over tens to hundreds of units, so later key
    blocks pass the reference of the running weights by more than its slack and the accumulated rows are rescaled;
    the softmax is close to a hard maximum.  A score of size |s| summed over d_h fp32 terms carries up to
    d_h 2^-24 |s| of rounding, which the exponential turns into that much relative error of a weight: the bar grows
    by that amount (a lost or doubled rescale would be off by the size of V itself)."""
    say("attention steep scores x%g" % gain)
    w = wl.small(T=900, d=512, K=400, L=1, dtype="bf16", seed=23, p=0.1)
    x = wl.layer_list(w)[0]
    q, k, v = wl.qkv(w, 2)
    q = (q.float() * gain).to(q.dtype)
    full = pa.fetch(pa.ada_select_full(x.to(DEV), w.tau))
    assert full["r"] > 256                                         # more than four key blocks
    idx = torch.as_tensor(full["idx"]).to(DEV)
    near = pa.ada_assign_nearest(x.to(DEV), idx)
    rows = np.asarray(full["idx"][:full["r"]])
    d_h = 256
    smax = max(float(np.abs(wl.as_f64(q)[rows, h * d_h:(h + 1) * d_h] @ wl.as_f64(k)[rows, h * d_h:(h + 1) * d_h].T).max())
               for h in range(2)) / np.sqrt(d_h)
    assert smax > 60.0
    vmax = float(np.abs(wl.as_f64(v)).max())
    tol = (parity.ATTN_TOL + smax * d_h * 2.0 ** -24) * max(1.0, vmax)
    for causal in (False, True):
        res = pa.ada_attention_compressed(q.to(DEV), k.to(DEV), v.to(DEV), 2, idx, near["assign"],
                                          flags=pa.FLAG_ATTN_CAUSAL if causal else 0)
        assert res["info"].cpu().tolist() == [full["r"], 0, 0, 0]
        ref = oracle.attention_compressed(wl.as_f64(q), wl.as_f64(k), wl.as_f64(v), 2, full["idx"],
                                          near["assign"].cpu().numpy(), flags=oracle.ATTN_CAUSAL if causal else 0)
        err = float(np.abs(res["out"].cpu().numpy().astype(np.float64) - ref).max())
        assert err <= tol, "steep scores x%g causal=%s: error %.3g, bar %.3g" % (gain, causal, err, tol)


def test_attention_into_a_strided_unaligned_output():
    """An output view whose rows start at odd float offsets (the vector stores of the bf16 kernel do not apply: the
    general kernel runs) gives the same rows as the contiguous output, and leaves the padding alone."""
    say("attention strided output")
    w = wl.small(T=400, d=256, K=60, L=1, dtype="bf16", seed=12, p=0.1)
    x = wl.layer_list(w)[0]
    q, k, v = (m.to(DEV) for m in wl.qkv(w, 2))
    sel = pa.ada_select_full(x.to(DEV), w.tau)
    r = int(sel["counts"][0].item())
    idx = sel["idx"][:r].clone()
    near = pa.ada_assign_nearest(x.to(DEV), idx)
    ref = pa.ada_attention_compressed(q, k, v, 2, idx, near["assign"])
    big = torch.full((w.T, 256 + 3), -7.0, dtype=torch.float32, device=DEV)
    view = big[:, 1:257]
    got = pa.ada_attention_compressed(q, k, v, 2, idx, near["assign"], out=view)
    assert got["info"].cpu().tolist() == ref["info"].cpu().tolist()
    assert np.abs(view.cpu().numpy() - ref["out"].cpu().numpy()).max() <= parity.ATTN_TOL * max(1.0, float(v.float().abs().max()))
    assert bool((big[:, 0] == -7.0).all()) and bool((big[:, 257:] == -7.0).all())
    parity.check_attention(q.cpu(), k.cpu(), v.cpu(), 2, idx.cpu().numpy(), near["assign"].cpu().numpy(),
                           view.cpu().numpy(), False, "strided output")


def test_attention_rejects_bad_sets_and_assignments():
    say("attention bad input")
    w = wl.small(T=200, d=128, K=20, L=1, dtype="bf16", seed=3)
    q, k, v = (m.to(DEV) for m in wl.qkv(w, 2))
    good_idx = torch.tensor([3, 50, 120], dtype=torch.int32, device=DEV)
    assign = torch.full((w.T,), 50, dtype=torch.int32, device=DEV)
    ok = pa.ada_attention_compressed(q, k, v, 2, good_idx, assign)
    assert ok["info"].cpu().tolist() == [3, 0, 0, 0]
    bad_assign = assign.clone(); bad_assign[7] = 51                 # not a member of R
    assert pa.ada_attention_compressed(q, k, v, 2, good_idx, bad_assign)["info"].cpu().tolist()[3] == 4
    bad_idx = torch.tensor([50, 3, 120], dtype=torch.int32, device=DEV)
    assert pa.ada_attention_compressed(q, k, v, 2, bad_idx, assign)["info"].cpu().tolist()[3] == 4
    zero = torch.zeros(1, dtype=torch.int32, device=DEV)
    assert pa.ada_attention_compressed(q, k, v, 2, good_idx, assign, r_dev=zero)["info"].cpu().tolist()[3] == 2


def test_attention_at_config2_size():
    say("attention config 2")
    w = wl.config(2)
    x = next(iter(wl.layers(w, 0, 1)))
    q, k, v = wl.qkv(w, 16)
    full = pa.fetch(pa.ada_select_full(x.to(DEV), w.tau))
    idx = torch.as_tensor(full["idx"]).to(DEV)
    near = pa.ada_assign_nearest(x.to(DEV), idx)
    res = pa.ada_attention_compressed(q.to(DEV), k.to(DEV), v.to(DEV), 16, idx, near["assign"])
    assert res["info"].cpu().tolist()[3] == 0
    parity.check_attention(q, k, v, 16, full["idx"], near["assign"].cpu().numpy(), res["out"].cpu().numpy(), False,
                           "config 2")
