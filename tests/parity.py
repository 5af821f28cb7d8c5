"""GPU-vs-oracle comparison helpers (the parity protocol).

Bars (stated by the benchmark spec and written out here):
  * gamma (max correlations): |gpu - oracle| <= GAMMA_TOL = 1e-4 absolute, the GPU accumulating in fp32 and the
    oracle in float64 on the same (bf16- or fp32-valued) inputs;
  * index sets, additions, removals and Gram-operation counts: bit-exact, except that a token whose ORACLE
    gamma lies within BAND = 1e-4 of 1 - tau^2 may take either decision; the oracle is then re-run with those
    decisions forced to the GPU's and everything must again be bit-exact.
Every cascade comparison is teacher-forced: the oracle consumes the same inherited set the GPU consumed.
"""
import numpy as np

import oracle
from paper_2605_03110_amd import workloads as wl

GAMMA_TOL = 1e-4
BAND = 1e-4


def thr_of(tau):
    return 1.0 - float(tau) * float(tau)


def check_full(x_cpu, tau, got, what=""):
    """got: ada.fetch() of ada_select_full."""
    X = wl.as_f64(x_cpu)
    T = X.shape[0]
    ref = oracle.select_full(X, tau)
    err = float(np.max(np.abs(got["gamma"].astype(np.float64) - ref["gamma"])))
    assert err <= GAMMA_TOL, "%s gamma error %.3g" % (what, err)
    band = np.abs(ref["gamma"] - thr_of(tau)) < BAND
    if band.any():
        force = -np.ones(T, dtype=np.int8)
        force[band] = got["mask"][band]
        ref = oracle.select_full(X, tau, force=force)
    assert np.array_equal(got["mask"], ref["mask"]), "%s mask differs at %s" % (
        what, np.flatnonzero(got["mask"] != ref["mask"])[:10])
    assert np.array_equal(got["idx"], ref["idx"]), what
    assert got["r"] == ref["r"], what
    return dict(ref=ref, gamma_err=err, n_band=int(band.sum()))


def check_cascade(x_cpu, tau, prev_idx, got, flags=0, what="", two_pass=False):
    """got: ada.fetch() of ada_cascade_step on the same prev_idx.  Both launch forms report Algorithm 1's own maxima
    (gamma^rep for an inherited token, gamma^cross over the valid representatives for any other), so `two_pass` only
    names the form in messages."""
    X = wl.as_f64(x_cpu)
    T = X.shape[0]
    prev_idx = np.asarray(prev_idx, dtype=np.int32)
    thr = thr_of(tau)
    in_gpu = np.zeros(T, dtype=np.int8)
    in_gpu[got["idx"]] = 1
    force = -np.ones(T, dtype=np.int8)
    ref = oracle.cascade_step(X, tau, prev_idx, flags=flags)
    for _ in range(4):   # forcing a representative's validity can move other tokens' gamma^cross into the band
        band = (np.abs(ref["gamma"] - thr) < BAND) & (force < 0)
        if not band.any():
            break
        force[band] = in_gpu[band]
        ref = oracle.cascade_step(X, tau, prev_idx, flags=flags, force=force)
    err = float(np.max(np.abs(got["gamma"].astype(np.float64) - ref["gamma"])))
    assert err <= GAMMA_TOL, "%s gamma error %.3g" % (what, err)
    for k in ("idx", "adds", "removes"):
        assert np.array_equal(got[k], ref[k]), "%s %s differs: gpu %s... oracle %s..." % (
            what, k, got[k][:8], ref[k][:8])
    assert got["gram_ops"] == ref["gram_ops"], what
    assert got["r"] == ref["r_new"] and got["n_adds"] == len(ref["adds"]) and got["n_removes"] == len(ref["removes"])
    return dict(ref=ref, gamma_err=err, n_band=int((force >= 0).sum()))


def check_assign(x_cpu, idx, got_assign, got_corr, what=""):
    """Section 2.3.  corr within GAMMA_TOL of the oracle; members of R map to themselves; for every other token
    the GPU's choice must be a member of R whose float64 |cosine| is within 2*GAMMA_TOL of the float64 maximum
    (several maximisers can be valid), and must equal the oracle's choice whenever the float64 runner-up is more
    than 2*GAMMA_TOL below the maximum (then the maximiser is unique at the kernel's accuracy)."""
    X = wl.as_f64(x_cpu)
    T = X.shape[0]
    idx = np.asarray(idx, dtype=np.int32)
    ref = oracle.assign_nearest(X, idx)
    err = float(np.max(np.abs(got_corr.astype(np.float64) - ref["corr"])))
    assert err <= GAMMA_TOL, "%s corr error %.3g" % (what, err)
    in_R = np.zeros(T, dtype=bool)
    in_R[idx] = True
    assert np.array_equal(got_assign[in_R], np.flatnonzero(in_R)), what
    assert in_R[got_assign].all(), "%s: assigned to a token outside R" % what
    Xn, _ = oracle.normalize(X)
    others = np.flatnonzero(~in_R)
    chosen = np.abs(np.einsum("ij,ij->i", Xn[others], Xn[got_assign[others]]))
    assert (chosen >= ref["corr"][others] - 2 * GAMMA_TOL).all(), what
    differ = others[got_assign[others] != ref["assign"][others]]
    for t in differ:          # only legitimate when another member of R is as close as the oracle's choice
        c = np.sort(np.abs(Xn[idx] @ Xn[t]))
        assert c[-1] - c[-2] <= 2 * GAMMA_TOL, "%s token %d: unique maximiser missed" % (what, t)
    return dict(ref=ref, corr_err=err, n_differ=int(len(differ)))


ATTN_TOL = 2e-5     # absolute, for value entries of unit scale; see the derivation next to the test


def check_attention(q, k, v, H, idx, assign, got_out, causal=False, what=""):
    """eq. (1): GPU output (float32) against the float64 oracle on the same (bf16- or fp32-valued) inputs."""
    ref = oracle.attention_compressed(wl.as_f64(q), wl.as_f64(k), wl.as_f64(v), H, idx, assign,
                                      flags=oracle.ATTN_CAUSAL if causal else 0)
    vmax = float(np.max(np.abs(wl.as_f64(v))))
    err = float(np.max(np.abs(got_out.astype(np.float64) - ref)))
    assert err <= ATTN_TOL * max(1.0, vmax), "%s attention error %.3g (|V| max %.3g)" % (what, err, vmax)
    return err
