"""Bookkeeping formulas of the paper, written out (TEST INFRASTRUCTURE ONLY).

Each function cites the equation or table that defines it.  Pure Python integers
and floats; nothing here is shared with the GPU library.
"""
from __future__ import annotations

from typing import Iterable, Sequence


def jaccard(a: Iterable[int], b: Iterable[int]) -> float:
    """eq. (3): |A n B| / |A u B| for two representative sets."""
    sa, sb = set(int(x) for x in a), set(int(x) for x in b)
    union = len(sa | sb)
    return len(sa & sb) / union if union else 1.0


def turnover(n_adds: int, n_removes: int, r_prev: int) -> float:
    """eq. (8): (|additions| + |removals|) / |R^(l)|, R^(l) being the set inherited FROM."""
    return (n_adds + n_removes) / r_prev


def gram_ops_full(T: int) -> int:
    """Table 6, "Independent" column: one layer of independent selection forms T*T Gram entries."""
    return T * T


def gram_ops_cascade(T: int, r: int, r_valid: int) -> int:
    """Algorithm 1, steps 3 and 7: an r x r Gram and a (T-r) x r_valid cross-Gram.
    Equals eq. (6)'s T*r (in entries) when no inherited representative is removed."""
    return r * r + (T - r) * r_valid


def cascade_cost_macs(T: int, r: int, d: int) -> int:
    """eq. (6): r^2 d + (T-r) r d = T r d."""
    return r * r * d + (T - r) * r * d


def selection_speedup(T: int, r: int) -> float:
    """eq. (7): T^2 d / (T r d) = T / r."""
    return T / r


def gram_savings(ops_cascade_per_layer: Sequence[int], T: int) -> float:
    """Table 6, "Savings": 1 - (cascade ops) / (independent ops), independent = L*T^2.
    The sequence holds one entry per layer, layer 0 (full selection) included."""
    L = len(ops_cascade_per_layer)
    return 1.0 - sum(int(x) for x in ops_cascade_per_layer) / (L * T * T)


def selection_cost_independent(L: int, T: int, d: int) -> int:
    """Section 6.6: L * T^2 * d."""
    return L * T * T * d


def selection_cost_cascade(L: int, T: int, d: int, r_bar: float) -> float:
    """Section 6.6: T d (T + (L-1) r_bar)."""
    return T * d * (T + (L - 1) * r_bar)


def attention_cost_compressed(L: int, r: float, d_h: int, heads: int) -> float:
    """FLOPs of the attention on r representatives over L layers: the two r x r x d_h products of eq. (1), at two
    FLOPs per multiply-add: L * 4 r^2 d_h * heads.  Section 6.6 writes the formula with a factor 2 but prints
    19.3 GFLOP for GPT-J, which is this count (the factor-2 form gives 9.6); the printed value is taken."""
    return float(L) * 4.0 * float(r) ** 2 * float(d_h) * float(heads)


def adapt_tau(tau: float, eta: float, kappa: float, eta_target: float, tau_min: float, tau_max: float) -> float:
    """Section 8.1, which states the rule in words only (low turnover: tighter threshold; high turnover: looser):
    tau moves by kappa * (eta_target - eta) and is clipped to [tau_min, tau_max]; a larger tau is the tighter
    threshold (1 - tau^2 falls, fewer representatives).  Python floats: IEEE double, one rounding per operation."""
    return min(max(tau + kappa * (eta_target - eta), tau_min), tau_max)
