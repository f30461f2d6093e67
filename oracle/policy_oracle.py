"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Plain Python/numpy statement of the cache-management policy arithmetic of Sec. 4.3, in the paper's
order and notation: the least-squares line of the time samples (the regression over
sampled token counts), Algorithm 1 (initial_cache_allocation, alloc_remaining), the ratio-keeping block
choice of Eq. 11 and the balance metric of Eq. 12-13.  Library routines (numpy.polyfit,
numpy.linalg.solve, fractions.Fraction) serve as steps.  It imports nothing from the GPU package.

Readings taken where the paper is silent:
  * T_kv_gen and T_load_kv are the fitted lines, intercept included, applied exactly as printed in
    Algorithm 1; a solution below zero is replaced by zero (and in step 2 the remaining memory then
    goes to the other block kind); block counts are rounded down to whole blocks.
  * Eq. 11 fixes a ratio, not a rule for ties: the next block is the kind that leaves the request's
    checkpoint share nearest the host share, and a tie goes to the checkpoint block (half the size).

Pins (tests/test_policy.py): the paper's worked example of Eq. 11, hand-computed instances of
Algorithm 1, the invariants the algorithm states (memory filled, times equal), brute force over
both block kinds for Eq. 11, exact rational arithmetic.  No function is "parity unpinned".
"""
from fractions import Fraction
import math

import numpy as np


def fit_line(n, t):
    """Least-squares line t ~ slope * n + offset and its R^2."""
    n, t = np.asarray(n, dtype=np.float64), np.asarray(t, dtype=np.float64)
    slope, offset = np.polyfit(n, t, 1)
    res = ((t - (slope * n + offset)) ** 2).sum()
    tot = ((t - t.mean()) ** 2).sum()
    return float(slope), float(offset), float(1.0 - res / tot) if tot > 0 else 1.0


def _T(line, n):
    return line[0] * n + line[1]


def initial_cache_allocation(T_load_w, T_kv_gen, T_load_kv, n_act_gpu):
    """Algorithm 1, step 1.  Lines are (slope, offset) pairs."""
    act_init, kv_init = 0.0, 0.0
    T_budget = T_load_w - _T(T_kv_gen, n_act_gpu)
    if T_budget >= 0:
        act_init = max(0.0, (T_budget - T_kv_gen[1]) / T_kv_gen[0])         # T_kv_gen(#ACT) = T_budget
    else:
        kv_init = max(0.0, (-T_budget - T_load_kv[1]) / T_load_kv[0])       # T_load_kv(#KV) = -T_budget
    return math.floor(act_init), math.floor(kv_init)


def alloc_remaining(act_init, kv_init, T_kv_gen, T_load_kv, M_host, S_weight, S_kv):
    """Algorithm 1, step 2: the 2 x 2 linear system over (#ACT, #KV)."""
    S_act = 0.5 * S_kv
    M_occupied = S_act * act_init + S_kv * kv_init
    M_remaining = M_host - S_weight - M_occupied
    if M_remaining <= 0:
        return 0, 0
    #   S_act * x + S_kv * y = M_remaining
    #   a * x - c * y        = e - b        (a x + b = c y + e)
    A = np.array([[S_act, S_kv], [T_kv_gen[0], -T_load_kv[0]]], dtype=np.float64)
    rhs = np.array([M_remaining, T_load_kv[1] - T_kv_gen[1]], dtype=np.float64)
    x, y = np.linalg.solve(A, rhs)
    if x < 0:
        x, y = 0.0, M_remaining / S_kv
    if y < 0:
        x, y = M_remaining / S_act, 0.0
    return math.floor(x), math.floor(y)


def host_block_allocation(T_load_w, T_kv_gen, T_load_kv, n_act_gpu, M_host, S_weight, S_kv):
    """Algorithm 1: returns (#ACT_Host, #KV_Host) and the four intermediate counts."""
    act_init, kv_init = initial_cache_allocation(T_load_w, T_kv_gen, T_load_kv, n_act_gpu)
    act_remain, kv_remain = alloc_remaining(act_init, kv_init, T_kv_gen, T_load_kv, M_host, S_weight, S_kv)
    return {"act_init": act_init, "kv_init": kv_init, "act_remain": act_remain, "kv_remain": kv_remain,
            "act_host": act_init + act_remain, "kv_host": kv_init + kv_remain}


def next_block_type(n_act, n_kv, act_host, kv_host):
    """Eq. 11: 'ACT' or 'KV', whichever leaves the checkpoint share of the request's blocks nearest
    act_host / (act_host + kv_host); exact rational arithmetic."""
    target = Fraction(act_host, act_host + kv_host)
    n1 = n_act + n_kv + 1
    dev_act = abs(Fraction(n_act + 1, n1) - target)
    dev_kv = abs(Fraction(n_act, n1) - target)
    return "ACT" if dev_act <= dev_kv else "KV"


def minibatch_balance(T_kv_gen, T_load_kv, n_act_mb, n_kv_mb):
    """Eq. 12 and 13: (balance, F_b)."""
    balance = _T(T_kv_gen, n_act_mb) / _T(T_load_kv, n_kv_mb)
    return balance, max(balance, 1.0 / balance)
