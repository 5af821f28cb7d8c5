"""The bookkeeping formulas (Jaccard eq. (3), turnover eq. (8), Gram-operation
counts of Table 6, the Section 6.6 cost model, eq. (7)) against the numbers the
paper prints.  The fixture holds only printed values with their citations."""
import os

import pytest

from oracle import metrics


def records(golden_dir, kind):
    out = []
    with open(os.path.join(golden_dir, "paper_bookkeeping.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            fields = [x.strip() for x in line.split("|")]
            if fields[0] == kind:
                out.append(fields[1:])
    assert out, kind
    return out


def test_independent_gram_ops_are_L_times_T_squared(golden_dir):
    for model, L, indep, casc, sav, _ in records(golden_dir, "gram_ops"):
        ops = int(L) * metrics.gram_ops_full(512)
        assert round(ops / 1e6, 2) == float(indep), model          # one operation = one Gram entry, T*T per layer


def test_savings_follow_from_the_tables_own_columns(golden_dir):
    for model, L, indep, casc, sav, _ in records(golden_dir, "gram_ops"):
        assert round(100 * (1 - float(casc) / float(indep))) == int(sav), model
    # and through the function, on synthetic per-layer counts that sum to the printed totals
    L, T = 28, 512
    per_layer = [T * T] + [int((3.51e6 - T * T) / (L - 1))] * (L - 1)
    assert round(100 * metrics.gram_savings(per_layer, T)) == 52


def test_cascade_size_chain_and_turnover_of_table_5(golden_dir):
    rows = records(golden_dir, "gptj_layer")
    r_prev = int(rows[0][1])
    for layer, r_casc, adds, rem, turn, _ in rows[1:]:
        adds, rem = int(adds), int(rem)
        assert r_prev + adds - rem == int(r_casc), layer            # |R_valid u R_new|
        assert abs(100 * metrics.turnover(adds, rem, r_prev) - int(turn)) <= 0.5, layer   # printed to the nearest percent
        r_prev = int(r_casc)


def test_turnover_denominator_is_the_inherited_set(golden_dir):
    for step, r_result, adds, rem, turn, _ in records(golden_dir, "turnover"):
        adds, rem = int(adds), int(rem)
        r_prev = int(r_result) - adds + rem
        assert round(100 * metrics.turnover(adds, rem, r_prev), 1) == float(turn), step


def test_jaccard_of_table_1(golden_dir):
    for model, ra, rb, inter, j, _ in records(golden_dir, "jaccard"):
        ra, rb, inter = int(ra), int(rb), int(inter)
        A = range(ra)
        B = range(ra - inter, ra - inter + rb)
        assert round(metrics.jaccard(A, B), 3) == float(j), (model, ra, rb)


def test_cost_model_and_speedup(golden_dir):
    for L, T, d, r_bar, printed, unit, _ in records(golden_dir, "cost_independent"):
        assert metrics.selection_cost_independent(int(L), int(T), int(d)) / 1e9 == pytest.approx(float(printed), rel=2e-3)
    for L, T, d, r_bar, printed, unit, _ in records(golden_dir, "cost_cascade"):
        got = metrics.selection_cost_cascade(int(L), int(T), int(d), float(r_bar)) / 1e9
        assert got == pytest.approx(float(printed), rel=1e-2)
    for L, r, dh, heads, printed, unit, _ in records(golden_dir, "cost_attention"):
        assert metrics.attention_cost_compressed(int(L), float(r), int(dh), int(heads)) / 1e9 == pytest.approx(float(printed), rel=2e-3)
    for L, T, d, r, printed, unit, _ in records(golden_dir, "speedup"):
        assert metrics.selection_speedup(int(T), int(r)) == pytest.approx(float(printed), rel=1e-2)


def test_eq6_identity_and_entry_count():
    for T, r, d in [(512, 69, 4096), (2048, 400, 4096), (16, 16, 3), (16, 1, 3)]:
        assert metrics.cascade_cost_macs(T, r, d) == T * r * d
        assert metrics.gram_ops_cascade(T, r, r) == T * r
        assert metrics.gram_ops_cascade(T, r, max(r - 1, 0)) == T * r - (T - r)
