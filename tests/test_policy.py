"""Cache-management policy arithmetic (Sec. 4.3): pins of the Python oracle against things other
than itself, then the C ABI (host-only functions of libhybridkv) against the oracle.  No GPU."""
import ctypes
import itertools
import math

import numpy as np
import pytest

from oracle import policy_oracle as po
from paper_2501_01792_amd import binding as hk


# ------------------------------------------------------------------ oracle pins
def test_oracle_next_block_paper_example():
    """Sec. 4.3, request block allocation: host ratio 3:1, five ACT and two KV blocks -> an ACT block."""
    assert po.next_block_type(5, 2, 3, 1) == "ACT"
    # the mirrored situation gives a KV block
    assert po.next_block_type(2, 5, 1, 3) == "KV"


@pytest.mark.parametrize("act_host,kv_host", [(3, 1), (1, 1), (2, 1), (178, 100), (1, 4), (5, 0), (0, 7)])
def test_oracle_next_block_keeps_the_ratio(act_host, kv_host):
    """Eq. 11 as an invariant: allocating block after block from an empty request, the request's ACT count
    never strays from its ideal share n * act_host / (act_host + kv_host) by a whole block."""
    n_act = n_kv = 0
    for n in range(1, 400):
        if po.next_block_type(n_act, n_kv, act_host, kv_host) == "ACT":
            n_act += 1
        else:
            n_kv += 1
        assert abs(n_act - n * act_host / (act_host + kv_host)) < 1.0
    # and it is the nearest choice at every step: brute force over both options
    for n_act, n_kv in itertools.product(range(12), range(12)):
        tgt = act_host / (act_host + kv_host)
        n1 = n_act + n_kv + 1
        dev = {"ACT": abs((n_act + 1) / n1 - tgt), "KV": abs(n_act / n1 - tgt)}
        got = po.next_block_type(n_act, n_kv, act_host, kv_host)
        assert dev[got] <= min(dev.values()) + 1e-12


def test_oracle_algorithm1_by_hand():
    """Algorithm 1 on numbers small enough for pencil and paper.
    T_kv_gen(n) = 2 n, T_load_kv(n) = 8 n, T_load_w = 100, #ACT_GPU = 20, S_KV = 4 (so S_ACT = 2),
    M_Host = 1000, S_weight = 380.
      step 1: T_budget = 100 - 40 = 60 >= 0 -> ACT_init = 30, KV_init = 0
      step 2: M_occupied = 60, M_remaining = 560; 2 x + 4 y = 560, 2 x = 8 y -> y = 46.67, x = 186.67
              -> 186 ACT, 46 KV blocks; totals 216 and 46."""
    r = po.host_block_allocation(100.0, (2.0, 0.0), (8.0, 0.0), 20, 1000.0, 380.0, 4.0)
    assert r == {"act_init": 30, "kv_init": 0, "act_remain": 186, "kv_remain": 46, "act_host": 216, "kv_host": 46}
    # weights load faster than the GPU-resident checkpoints regenerate: the PCIe link would idle, KV blocks fill it
    #   T_budget = 10 - 40 = -30 -> KV_init = 30 / 8 = 3.75 -> 3; M_remaining = 1000 - 380 - 12 = 608
    #   2 x + 4 y = 608, 2 x = 8 y -> y = 50.67, x = 202.67
    r = po.host_block_allocation(10.0, (2.0, 0.0), (8.0, 0.0), 20, 1000.0, 380.0, 4.0)
    assert r == {"act_init": 0, "kv_init": 3, "act_remain": 202, "kv_remain": 50, "act_host": 202, "kv_host": 53}


def test_oracle_algorithm1_step1_with_intercepts_by_hand():
    """Step 1 of Algorithm 1 with lines that do not pass through the origin, both branches, by hand:
    T_kv_gen(n) = 2 n + 6, T_load_kv(n) = 8 n + 4, #ACT_GPU = 20 (so the GPU-resident checkpoints take 46).
      T_load_w = 100: T_budget = 54 >= 0 -> 2 n + 6 = 54 -> ACT_init = 24 (a sign slip on the intercept gives 30)
      T_load_w = 10:  T_budget = -36 < 0 -> 8 n + 4 = 36 -> KV_init = 4    (a sign slip gives 5)
      T_load_w = 49:  T_budget = 3 < the intercept 6 -> no block count gives so short a time: ACT_init = 0
      T_load_w = 44:  T_budget = -2, shorter than T_load_kv(0) = 4 -> KV_init = 0."""
    gen, load = (2.0, 6.0), (8.0, 4.0)
    assert po.initial_cache_allocation(100.0, gen, load, 20) == (24, 0)
    assert po.initial_cache_allocation(10.0, gen, load, 20) == (0, 4)
    assert po.initial_cache_allocation(49.0, gen, load, 20) == (0, 0)
    assert po.initial_cache_allocation(44.0, gen, load, 20) == (0, 0)
    # fractional solutions round down to whole blocks: T_budget = 55 -> n = 24.5; T_budget = -39 -> n = 4.375
    assert po.initial_cache_allocation(101.0, gen, load, 20) == (24, 0)
    assert po.initial_cache_allocation(7.0, gen, load, 20) == (0, 4)
    # the whole algorithm on the first instance: S_KV = 4, M_Host = 1000, S_weight = 380
    #   M_occupied = 2 * 24 = 48, M_remaining = 572; 2 x + 4 y = 572 and 2 x + 6 = 8 y + 4
    #   -> x = 4 y - 1 -> 12 y = 574 -> y = 47.83, x = 190.33 -> 190 ACT, 47 KV; totals 214 and 47
    r = po.host_block_allocation(100.0, gen, load, 20, 1000.0, 380.0, 4.0)
    assert r == {"act_init": 24, "kv_init": 0, "act_remain": 190, "kv_remain": 47, "act_host": 214, "kv_host": 47}


def test_oracle_algorithm1_step1_closes_the_time_gap():
    """The property step 1 states, on its real-valued solution (recovered here to within the floor): the
    regeneration time of ACT_init blocks equals T_budget, or the load time of KV_init blocks equals -T_budget;
    exactly one of the two is non-zero unless the gap is shorter than the line's intercept."""
    rng = np.random.default_rng(11)
    seen = set()
    for _ in range(400):
        gen = (rng.uniform(0.1, 3.0), rng.uniform(0.0, 5.0))
        load = (rng.uniform(0.5, 12.0), rng.uniform(0.0, 5.0))
        n_gpu = int(rng.integers(0, 100))
        T_w = rng.uniform(0.0, 400.0)
        T_budget = T_w - (gen[0] * n_gpu + gen[1])
        act, kv = po.initial_cache_allocation(T_w, gen, load, n_gpu)
        assert act >= 0 and kv >= 0 and (act == 0 or kv == 0)
        if T_budget >= 0:
            assert kv == 0
            if T_budget >= gen[1]:
                # floor: T_kv_gen(act) <= T_budget < T_kv_gen(act + 1)
                assert gen[0] * act + gen[1] <= T_budget + 1e-9 < gen[0] * (act + 1) + gen[1] + 1e-9
                seen.add("act")
            else:
                assert act == 0
                seen.add("act0")
        else:
            assert act == 0
            if -T_budget >= load[1]:
                assert load[0] * kv + load[1] <= -T_budget + 1e-9 < load[0] * (kv + 1) + load[1] + 1e-9
                seen.add("kv")
            else:
                assert kv == 0
                seen.add("kv0")
    assert seen == {"act", "act0", "kv", "kv0"}


def test_oracle_algorithm1_invariants():
    """What step 2 states must hold for its real-valued solution (re-derived here with numpy's solver on
    the system as printed): the memory is filled exactly and the two times are equal; rounding down to
    whole blocks wastes less than one block of each kind."""
    rng = np.random.default_rng(7)
    for _ in range(200):
        a, c = rng.uniform(0.5, 3.0), rng.uniform(2.0, 12.0)
        b, e = rng.uniform(0.0, 5.0), rng.uniform(0.0, 5.0)
        S_kv = rng.uniform(2.0, 8.0)
        M_rem = rng.uniform(200.0, 900.0)
        A = np.array([[S_kv / 2, S_kv], [a, -c]])
        x, y = np.linalg.solve(A, [M_rem, e - b])
        if x < 0 or y < 0:
            continue
        assert abs(S_kv / 2 * x + S_kv * y - M_rem) < 1e-9 * M_rem
        assert abs((a * x + b) - (c * y + e)) < 1e-9 * (a * x + b)
        got = po.alloc_remaining(0, 0, (a, b), (c, e), M_rem, 0.0, S_kv)
        assert got == (math.floor(x), math.floor(y))
        gx, gy = got
        waste = M_rem - (S_kv / 2 * gx + S_kv * gy)
        assert 0 <= waste < 1.5 * S_kv


def test_oracle_fit_line_and_balance():
    n = np.array([128, 256, 512, 1024, 2048, 4096], dtype=np.float64)
    s, o, r2 = po.fit_line(n, 0.25 * n + 3.0)
    assert abs(s - 0.25) < 1e-12 and abs(o - 3.0) < 1e-9 and abs(r2 - 1.0) < 1e-12
    # closed form of the slope: cov / var
    t = np.array([40.0, 70.0, 150.0, 260.0, 540.0, 1010.0])
    s, o, r2 = po.fit_line(n, t)
    assert abs(s - np.cov(n, t, bias=True)[0, 1] / n.var()) < 1e-12
    assert 0.99 < r2 <= 1.0
    bal, cost = po.minibatch_balance((2.0, 0.0), (8.0, 0.0), 40, 10)
    assert bal == 1.0 and cost == 1.0
    bal, cost = po.minibatch_balance((2.0, 0.0), (8.0, 0.0), 40, 20)
    assert bal == 0.5 and cost == 2.0
    bal2, cost2 = po.minibatch_balance((2.0, 0.0), (8.0, 0.0), 160, 20)
    assert bal2 == 2.0 and cost2 == 2.0                          # F_b treats both directions of imbalance alike


# ------------------------------------------------------------------ C ABI against the oracle
def test_c_next_block_type_matches_oracle():
    assert hk.next_block_type(5, 2, 3, 1) == "ACT"
    rng = np.random.default_rng(8)
    for _ in range(3000):
        n_act, n_kv = (int(v) for v in rng.integers(0, 500, 2))
        act_host, kv_host = (int(v) for v in rng.integers(0, 300, 2))
        if act_host + kv_host == 0:
            continue
        assert hk.next_block_type(n_act, n_kv, act_host, kv_host) == po.next_block_type(n_act, n_kv, act_host, kv_host)
    L = hk.lib()
    assert L.hk_next_block_type(-1, 0, 1, 1) == hk.HK_ERR_SHAPE
    assert L.hk_next_block_type(0, 0, 0, 0) == hk.HK_ERR_SHAPE
    assert L.hk_next_block_type(1 << 40, 0, 1, 1) == hk.HK_ERR_SHAPE


def test_c_host_block_allocation_matches_oracle():
    rng = np.random.default_rng(9)
    cases = [(100.0, (2.0, 0.0), (8.0, 0.0), 20, 1000.0, 380.0, 4.0), (10.0, (2.0, 0.0), (8.0, 0.0), 20, 1000.0, 380.0, 4.0)]
    for _ in range(500):
        cases.append((rng.uniform(0, 200), (rng.uniform(0.1, 3), rng.uniform(0, 5)), (rng.uniform(0.5, 12), rng.uniform(0, 5)),
                      float(rng.integers(0, 200)), rng.uniform(500, 1e5), rng.uniform(0, 600), rng.uniform(1, 16)))
    for c in cases:
        assert hk.host_block_allocation(*c) == po.host_block_allocation(*c), c
    # OPT-30B-sized instance in bytes and milliseconds: 16-token blocks, d = 7168, 48 layers
    S_kv = 16 * 4 * 7168 * 48
    c = (31.85, (0.0045, 0.02), (0.018, 0.01), 1024.0, 800e9, 60e9, float(S_kv))
    assert hk.host_block_allocation(*c) == po.host_block_allocation(*c)
    # lines with intercepts, both branches of step 1 (the hand-computed instances of the oracle's pin)
    for T_w in (100.0, 10.0, 49.0, 44.0, 101.0, 7.0):
        c = (T_w, (2.0, 6.0), (8.0, 4.0), 20, 1000.0, 380.0, 4.0)
        assert hk.host_block_allocation(*c) == po.host_block_allocation(*c), c
    p = hk.hk_alloc_params(1.0, hk.hk_line(0.0, 0.0), hk.hk_line(1.0, 0.0), 0.0, 10.0, 0.0, 1.0)
    r = hk.hk_alloc_result()
    assert hk.lib().hk_host_block_allocation(ctypes.byref(p), ctypes.byref(r)) == hk.HK_ERR_SHAPE   # zero slope
    assert hk.lib().hk_host_block_allocation(None, ctypes.byref(r)) == hk.HK_ERR_NULL
    # block counts that do not fit 62 bits are refused instead of being cast (huge memory, tiny blocks or slopes)
    for bad in (hk.hk_alloc_params(1.0, hk.hk_line(1.0, 0.0), hk.hk_line(1.0, 0.0), 0.0, 1e300, 0.0, 1.0),
                hk.hk_alloc_params(1e30, hk.hk_line(1e-300, 0.0), hk.hk_line(1.0, 0.0), 0.0, 10.0, 0.0, 1.0),
                hk.hk_alloc_params(0.0, hk.hk_line(1.0, 0.0), hk.hk_line(1e-300, 0.0), 1e30, 10.0, 0.0, 1.0),
                hk.hk_alloc_params(1.0, hk.hk_line(1.0, 0.0), hk.hk_line(1.0, 0.0), 0.0, 1e19, 0.0, 1e-3)):
        assert hk.lib().hk_host_block_allocation(ctypes.byref(bad), ctypes.byref(r)) == hk.HK_ERR_SHAPE


def test_c_fit_line_and_balance_match_oracle():
    rng = np.random.default_rng(10)
    for _ in range(50):
        n = np.sort(rng.uniform(16, 1e5, 12))
        t = rng.uniform(0.001, 0.01) * n + rng.uniform(0, 3) + rng.normal(0, 0.05, 12)
        got, ref = hk.fit_line(n, t), po.fit_line(n, t)
        np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-9)
        lines = ((got[0], abs(got[1]) + 0.1), (rng.uniform(0.001, 0.05), rng.uniform(0.1, 2)))
        a, k = rng.uniform(1, 1e4), rng.uniform(1, 1e4)
        np.testing.assert_allclose(hk.minibatch_balance(*lines, a, k), po.minibatch_balance(*lines, a, k), rtol=1e-12)
    with pytest.raises(hk.HybridKVError):
        hk.fit_line([3.0, 3.0, 3.0], [1.0, 2.0, 3.0])
    with pytest.raises(hk.HybridKVError):
        hk.minibatch_balance((1.0, 0.0), (1.0, 0.0), 5.0, 0.0)           # zero load time: no ratio
