"""Pins for oracle/scheduler.py and oracle/bubbles.py: hand-computed example, exhaustive invariants, closed
forms, and a discrete-event simulation of the 1F1B pipeline written independently of the closed form."""
import itertools
import os

import numpy as np
import pytest

import synth_inputs as S
from oracle import bubbles as B
from oracle import scheduler as K

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_zero_count_and_window():
    assert K.zero_count([]) == 0
    assert K.zero_count([3, 0, 0]) == 2 and K.zero_count([0, 0, 1]) == 0 and K.zero_count([0, 0, 0]) == 3
    bm = K.BubbleMonitor(4)
    assert [bm.push(c) for c in (5, 0, 0, 0, 0, 0, 2, 0)] == [0, 1, 2, 3, 4, 4, 0, 1]   # saturates at the window


def test_alg1_hand_example():
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLD, "alg1_worked_example.txt")) if l[0] != "#"]
    pool = 0
    for zc, want_pool, want_grant, want_status in rows:
        pool, grant, status = K.alg1_step(zc, pool, 2, 5, 2, 1, 2, 8, 64, 1)
        assert (pool, grant, status) == (want_pool, want_grant, want_status)


def test_alg1_phase_invariants_exhaustive():
    # every Z_c trace of length <= 6 over {0..5}, a small parameter grid
    for alpha, beta, m, ll, ul, t0, gn, gd in ((0, 2, 1, 4, 16, 1, 2, 1), (1, 3, 2, 6, 40, 2, 3, 2), (2, 2, 3, 9, 9, 3, 2, 1)):
        for n in range(1, 7):
            for trace in itertools.product(range(6), repeat=n):
                pool = 0
                for zc in trace:
                    prev = pool
                    pool, grant, status = K.alg1_step(zc, pool, alpha, beta, gn, gd, m, ll, ul, t0)
                    assert (grant == 0 and pool == 0) == (zc <= alpha) or (zc > alpha and pool // m == 0)
                    assert (status == K.IDLE) == (zc > beta)
                    if zc <= alpha:
                        assert pool == 0 and grant == 0 and status == K.BUSY
                    elif zc <= beta:
                        assert pool == min(ll, max(prev, t0) * gn // gd) and grant == pool // m <= ll // m
                    else:
                        assert pool == min(ul, max(prev, t0) * gn // gd) and grant == pool // m <= ul // m


def test_alg1_constant_phase_closed_form():
    # k periods in the stable phase from an empty pool: pool = min(UL, T0 * gamma^k)
    pool = 0
    for k in range(1, 12):
        pool, grant, _ = K.alg1_step(99, pool, 1, 4, 2, 1, 1, 50, 1000, 3)
        assert pool == min(1000, 3 * 2 ** k) and grant == pool


def test_kb_release_rules():
    assert K.kb_release([3, 3, 3], 7) == (2, 1)
    assert K.kb_release([5, 1, 1], 4) == (0, 4)          # head of line blocks
    assert K.kb_release([], 10) == (0, 10)
    assert K.kb_release([2, 2], 0) == (0, 0)
    assert K.kb_release([0, 0], 0) == (2, 0)
    # brute force: released prefix is the longest whose running sum fits
    for costs in itertools.product(range(4), repeat=4):
        for bal in range(8):
            n, left = K.kb_release(list(costs), bal)
            assert sum(costs[:n]) + left == bal and (n == 4 or costs[n] > left)


def test_online_pull_and_principles():
    assert K.online_pull_ok(K.IDLE, 1, 10, 10)
    assert not K.online_pull_ok(K.BUSY, 1, 10, 1)
    assert not K.online_pull_ok(K.IDLE, 0, 10, 1)
    assert not K.online_pull_ok(K.IDLE, 1, 9, 10)
    assert K.principle_1([30, 9], 40) and not K.principle_1([30, 10], 40)
    assert K.principle_2(5, 6) and not K.principle_2(6, 6)


def test_run_trace_releases_only_with_tokens():
    counts = [4, 0, 0, 0, 0, 0, 0, 3, 0, 0, 0]
    costs = [2] * 30
    rows = K.run_trace(counts, costs, 8, 1, 3, 2, 1, 1, 4, 16, 1)
    assert [r[0] for r in rows] == [0, 1, 2, 3, 4, 5, 6, 0, 1, 2, 3]
    assert [r[1] for r in rows] == [0, 0, 2, 4, 8, 16, 16, 0, 0, 2, 4]
    assert [r[4] for r in rows] == [0, 0, 1, 2, 4, 8, 8, 0, 0, 1, 2]
    for zc, pool, grant, status, n in rows:
        assert 2 * n <= grant


# ---------------------------------------------------------------- bubble model
def test_dp_and_tp_closed_values():
    from oracle.decoder import n_params
    n = n_params(S.DP_DECODER)
    (site, ns), = B.dp_bubbles(n, 2, 50_000_000_000)
    assert n * 2 == 248_879_616 and ns == 4_977_592          # 248.9 MB at 50 GB/s = 4.98 ms
    (_, ns_ring), = B.dp_bubbles(n, 2, 50_000_000_000, ring_factor_num=6, ring_factor_den=4)   # 2(N-1)/N, N=4
    assert ns_ring == 7_466_388
    c = S.TP_DECODER
    tp = B.tp_bubbles(c["n_layers"], c["batch"] * c["seq"], c["d_model"], 2, c["bw_bytes_per_s"])
    assert len(tp) == 96 and all(ns == 1_342_177 for _, ns in tp)   # 67,108,864 B at 50 GB/s
    assert tp[0][0] == "fwd0.attn_out" and tp[48][0] == "bwd23.mlp_up_dgrad" and tp[-1][0] == "bwd0.qkv_dgrad"


def simulate_1f1b(p, m, tf, tb):
    """Event simulation of all stages: F(s,k) needs F(s-1,k); B(s,k) needs B(s+1,k) (and F(s,k) on the last
    stage); each stage runs its ops in 1F1B order.  Returns per stage the list of (op, start, end)."""
    order = [B.pp_1f1b_ops(s, p, m) for s in range(p)]
    done, pos, free, log = {}, [0] * p, [0] * p, [[] for _ in range(p)]
    progressed = True
    while progressed:
        progressed = False
        for s in range(p):
            if pos[s] == len(order[s]):
                continue
            kind, k = order[s][pos[s]]
            if kind == "F":
                dep = done.get(("F", s - 1, k)) if s > 0 else 0
            else:
                dep = done.get(("B", s + 1, k)) if s < p - 1 else done.get(("F", s, k))
            if dep is None:
                continue
            start = max(dep, free[s])
            end = start + (tf if kind == "F" else tb)
            done[(kind, s, k)] = end
            free[s] = end
            log[s].append(((kind, k), start, end))
            pos[s] += 1
            progressed = True
    assert all(pos[s] == len(order[s]) for s in range(p))
    return log


@pytest.mark.parametrize("p,m,tf,tb", [(4, 8, 100, 200), (4, 8, 7, 19), (3, 3, 5, 5), (2, 6, 11, 30), (5, 9, 3, 8)])
def test_pp_closed_form_against_event_simulation(p, m, tf, tb):
    log = simulate_1f1b(p, m, tf, tb)
    t_end = max(l[-1][2] for l in log)
    assert t_end == (m + p - 1) * (tf + tb)
    for s in range(p):
        gaps, t = [], 0
        for op, start, end in log[s]:
            if start > t:
                gaps.append((("before", op), start - t))
            t = end
        if t_end > t:
            gaps.append((("end", None), t_end - t))
        assert gaps == B.pp_1f1b_bubbles(s, p, m, tf, tb), s
        assert sum(g for _, g in gaps) == (p - 1) * (tf + tb)


# ---- bucketed gradient exchange beside backward (data parallel, overlapped)
def test_dp_buckets_rule():
    assert B.dp_gradient_buckets([10, 10, 10, 10, 10], 25) == [[0, 1, 2], [3, 4]]
    assert B.dp_gradient_buckets([10, 10, 10, 10, 10], 20) == [[0, 1], [2, 3], [4]]
    assert B.dp_gradient_buckets([100, 1, 1], 25) == [[0], [1, 2]]                # an oversized group closes its bucket
    assert B.dp_gradient_buckets([1, 100, 1], 25) == [[0, 1], [2]]
    assert B.dp_gradient_buckets([3, 4], 10 ** 9) == [[0, 1]]                     # cap never reached: one bucket
    assert B.dp_gradient_buckets([], 5) == []
    for sizes in itertools.product([1, 7, 30], repeat=5):
        for cap in (1, 8, 25, 64):
            bk = B.dp_gradient_buckets(list(sizes), cap)
            assert [i for b in bk for i in b] == list(range(5))                   # a partition that keeps the order
            for b in bk[:-1]:
                tot = sum(sizes[i] for i in b)
                assert tot >= cap and tot - sizes[b[-1]] < cap                    # closed exactly when the cap is reached


def simulate_link(ready, dur, end):
    """Tick-by-tick simulation of one link that sends the buckets in order, one at a time."""
    t, k, left, busy = 0, 0, 0, False
    n = len(ready)
    while k < n:
        if not busy and ready[k] <= t:
            busy, left = True, dur[k]
        if busy and left == 0:
            busy = False
            k += 1
            continue
        if busy:
            left -= 1
        t += 1
    return max(0, t - end)


def test_dp_overlapped_wait_against_tick_simulation_and_closed_forms():
    rng = np.random.default_rng(77)
    for _ in range(300):
        n = int(rng.integers(1, 6))
        ready = sorted(int(v) for v in rng.integers(0, 40, n))
        dur = [int(v) for v in rng.integers(0, 15, n)]
        end = ready[-1] + int(rng.integers(0, 10))
        got = B.dp_overlapped_wait(ready, dur, end)
        assert got == simulate_link(ready, dur, end), (ready, dur, end)
        # max-plus closed form of the recursion: the last bucket arrives at max_j (ready_j + sum of dur from j on)
        assert got == max(0, max(ready[j] + sum(dur[j:]) for j in range(n)) - end)
        assert got <= sum(dur)                                      # never worse than no overlap at all
        assert got >= max(0, ready[-1] + dur[-1] - end)             # the last bucket cannot start before it is ready
    # nothing overlaps when every gradient is final only at the end of backward: the whole exchange is exposed
    assert B.dp_overlapped_wait([50, 50, 50], [7, 8, 9], 50) == 24
    # everything final at time 0: the exchange has had the whole of backward to itself
    assert B.dp_overlapped_wait([0, 0, 0], [7, 8, 9], 20) == 4 and B.dp_overlapped_wait([0, 0, 0], [7, 8, 9], 30) == 0
    # an exchange that takes no time exposes nothing
    assert B.dp_overlapped_wait([3, 9, 12], [0, 0, 0], 12) == 0
    # a slow link behind a fast backward: the backlog of the earlier buckets delays the last one
    assert B.dp_overlapped_wait([10, 20, 30], [100, 100, 100], 30) == 10 + 300 - 30
    # one bucket = the unbucketed exchange of the configuration
    n_params = 124_439_808
    (_, whole), = B.dp_bubbles(n_params, 2, 50_000_000_000)
    assert B.dp_overlapped_wait([1000], [whole], 1000) == whole


# ---- concurrent filling with feedback
def test_feedback_share_rule_and_its_closed_forms():
    P = K.PPM
    assert K.feedback_share(200_000, 1_021, 1_000, 20_000, 50_000) == 100_000       # 2.1 % longer: halved
    assert K.feedback_share(200_000, 1_020, 1_000, 20_000, 50_000) == 250_000       # exactly at the threshold: not longer
    assert K.feedback_share(980_000, 900, 1_000, 20_000, 50_000) == P               # capped
    assert K.feedback_share(1, 2_000, 1_000, 20_000, 50_000) == 0                   # halving reaches zero
    # k good iterations from zero: min(cap, k * add); then h bad ones: floor division by 2^h
    s = 0
    for k in range(1, 30):
        s = K.feedback_share(s, 100, 100, 0, 70_000, 600_000)
        assert s == min(600_000, 70_000 * k)
    for h in range(1, 8):
        s = K.feedback_share(s, 101, 100, 0, 70_000, 600_000)
        assert s == 600_000 >> h
    # exhaustive: never outside [0, cap], monotone in the iteration time
    for share in range(0, 1_000_001, 125_000):
        prev = None
        for step in range(90, 121):
            v = K.feedback_share(share, step, 100, 50_000, 125_000)
            assert 0 <= v <= P
            assert prev is None or v <= prev
            prev = v


def test_feedback_holds_a_linear_plant_near_its_threshold():
    """Plant: an iteration takes ref * (1 + kappa * share).  The share climbs by `add` until the threshold share
    eps / kappa is passed, is halved, and climbs again: the slowdown never exceeds eps + kappa * add, and the
    long-run share stays between a third of the threshold share and the threshold share plus one increment."""
    ref, eps, add = 100_000_000, 20_000, 10_000
    for kappa_ppm in (100_000, 400_000, 900_000):            # slowdown per unit share
        star = eps * K.PPM // kappa_ppm                      # share at which the threshold is met
        share, shares, worst = 0, [], 0
        for _ in range(2000):
            step = ref + ref * kappa_ppm // K.PPM * share // K.PPM
            worst = max(worst, step)
            share = K.feedback_share(share, step, ref, eps, add)
            shares.append(share)
        assert worst <= ref + ref * (eps + kappa_ppm * add // K.PPM) // K.PPM + 1
        tail = shares[500:]
        assert max(tail) <= min(K.PPM, star + add)
        if star + add < K.PPM:
            assert sum(tail) / len(tail) >= star / 3


def test_concurrent_account():
    assert K.concurrent_account(0, 100_000, 25_000, 10 ** 9) == 2_500
    assert K.concurrent_account(0, 1_000_000, 25_000, 10 ** 9) == 25_000            # full share: the whole period
    assert K.concurrent_account(190_000, 1_000_000, 25_000, 200_000) == 200_000     # burst cap
    assert K.concurrent_account(7, 0, 25_000, 200_000) == 7                         # no share, nothing gained
    # n busy periods at a constant share: floor per period, so n * floor(period * share)
    b = 0
    for n in range(1, 50):
        b = K.concurrent_account(b, 333_333, 25_000, 10 ** 9)
        assert b == n * (25_000 * 333_333 // K.PPM)

