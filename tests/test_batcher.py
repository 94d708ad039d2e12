"""Dynamic-window batching (Section 3.2, Eq. 1): pins of the oracle, then the native queue against it."""
import math
import threading

import numpy as np
import pytest

from oracle import batcher_oracle as BO
from paper_2603_18464_amd import binding as B


# ---- the oracle against what Eq. 1 fixes ---------------------------------------------------------------

def test_trigger_truth_table():
    # (|Q|, B, t_now, t_first, T_max) -> the two clauses of Eq. 1, separately and together
    assert BO.trigger(4, 4, 0.0, 0.0, 1.0)            # size clause alone
    assert BO.trigger(9, 4, 0.0, 0.0, 1.0)
    assert not BO.trigger(3, 4, 0.999, 0.0, 1.0)      # neither
    assert BO.trigger(3, 4, 1.0, 0.0, 1.0)            # waiting clause alone, boundary is inclusive (>=)
    assert BO.trigger(1, 4, 5.5, 4.0, 1.5)
    assert not BO.trigger(1, 4, 5.4, 4.0, 1.5)
    assert not BO.trigger(0, 4, 100.0, 0.0, 1.0)      # nothing to run


def test_hand_worked_trace():
    """B = 3, T_max = 10 ms.  Requests 0..6 arrive at 0, 1, 2, 3, 4, 30, 31 ms; polls every 5 ms from 0 to 45.
    By hand: poll 0 sees {0} (waited 0) -> nothing; poll 5 sees {0,1,2,3,4}: size clause -> [0,1,2]; poll 10 sees
    {3,4}: oldest arrived at 3, waited 7 -> nothing; poll 15: waited 12 -> [3,4]; polls 20, 25 empty; poll 30
    sees {5}; poll 35 sees {5,6}, waited 5; poll 40: waited 10 -> [5,6]; poll 45 empty."""
    arr = [0, 1, 2, 3, 4, 30, 31]
    ev = []
    a = 0
    for p in range(0, 50, 5):
        while a < len(arr) and arr[a] <= p:
            ev.append(("push", arr[a] * 1e-3, a, 10))
            a += 1
        ev.append(("poll", p * 1e-3))
    assert BO.simulate(ev, 3, 10e-3) == [(5e-3, [0, 1, 2]), (15e-3, [3, 4]), (40e-3, [5, 6])]


def test_burst_and_token_capacity():
    ev = [("push", 0.0, i, 100) for i in range(10)] + [("poll", 0.0)] * 3 + [("poll", 0.5), ("poll", 1.0)]
    # 10 requests at once, B = 4: two full batches at once, the last two only when they have waited T_max
    assert BO.simulate(ev, 4, 1.0) == [(0.0, [0, 1, 2, 3]), (0.0, [4, 5, 6, 7]), (1.0, [8, 9])]
    # capacity of 250 tokens: the size clause still fires on |Q| >= 4, but only two requests fit
    got = BO.simulate(ev, 4, 1.0, max_tokens=250)
    assert got[:3] == [(0.0, [0, 1]), (0.0, [2, 3]), (0.0, [4, 5])]
    # conservation and order: every request exactly once, in arrival order, never more than B
    flat = [r for _, b in got for r in b]
    assert flat == sorted(flat) and len(set(flat)) == len(flat)
    assert BO.deadline([], 1.0) == math.inf and BO.deadline([2.0, 3.0], 1.0) == 3.0


def test_t_max_zero_and_huge_batch_degenerate_cases():
    ev = []
    for i in range(5):
        ev += [("push", float(i), i, 1), ("poll", float(i))]
    assert BO.simulate(ev, 8, 0.0) == [(float(i), [i]) for i in range(5)]        # T_max = 0: never wait
    assert BO.simulate(ev, 1, 1e9) == [(float(i), [i]) for i in range(5)]        # B = 1: never wait either
    assert BO.simulate(ev, 8, 1e9) == []                                         # neither clause can fire


# ---- the native queue against the oracle ----------------------------------------------------------------

def random_trace(seed, n_req, rate, poll_dt, burstiness):
    g = np.random.default_rng(seed)
    gaps = g.exponential(1.0 / rate, n_req) * g.choice([0.0, 1.0, 4.0], n_req, p=burstiness)
    t_arr = np.cumsum(gaps)
    toks = g.integers(1, 300, n_req)
    ev, a, t = [], 0, 0.0
    while a < n_req or t < t_arr[-1] + 2.0:
        while a < n_req and t_arr[a] <= t:
            ev.append(("push", float(t_arr[a]), a, int(toks[a])))
            a += 1
        ev.append(("poll", t))
        if g.random() < 0.3:
            ev.append(("poll", t))            # back-to-back polls
        t += poll_dt * (0.5 + g.random())
    return ev


def run_native(ev, Bt, T_max, max_tokens):
    q = B.Batcher(Bt, T_max, max_tokens)
    out = []
    for e in ev:
        if e[0] == "push":
            n_patch = e[3] // 2
            q.push(e[2], n_patch, e[3] - n_patch, e[1])
        else:
            got = q.poll(e[1], e[2] if len(e) > 2 else None)
            if got:
                out.append((e[1], [r[0] for r in got]))
    left = len(q)
    q.close()
    return out, left


@pytest.mark.parametrize("seed,Bt,T_max,max_tokens", [(1, 8, 0.05, 0), (2, 64, 0.02, 0), (3, 16, 0.0, 0),
                                                     (4, 4, 0.5, 700), (5, 128, 0.01, 9000), (6, 1, 1.0, 0)])
def test_native_queue_equals_oracle_on_random_traces(seed, Bt, T_max, max_tokens):
    ev = random_trace(seed, 600, rate=400.0, poll_dt=0.004, burstiness=[0.5, 0.4, 0.1])
    want = BO.simulate(ev, Bt, T_max, max_tokens)
    got, left = run_native(ev, Bt, T_max, max_tokens)
    assert got == want
    assert left == 0 and sum(len(b) for _, b in got) == 600          # the trace polls long enough to empty Q
    assert max(len(b) for _, b in got) <= Bt


def test_poll_capacity_limits_the_batch_not_the_trigger():
    """A caller with fewer free places than the target batch (continuous batching): the rule fires as before,
    the batch is cut to what can be taken, the rest waits with its own arrival times."""
    ev = [("push", 0.0, i, 10) for i in range(6)] + [("poll", 0.0, 2), ("poll", 0.0, 1), ("poll", 0.0, 8),
                                                      ("poll", 0.5, 8), ("poll", 1.0, 1), ("poll", 1.0, 8)]
    # B = 4: |Q| = 6 >= 4 fires, take 2; |Q| = 4 fires, take 1; |Q| = 3: wait; at t = 1.0 the oldest has waited T_max
    want = [(0.0, [0, 1]), (0.0, [2]), (1.0, [3]), (1.0, [4, 5])]
    assert BO.simulate(ev, 4, 1.0) == want
    got, left = run_native(ev, 4, 1.0, 0)
    assert got == want and left == 0
    g = np.random.default_rng(11)
    ev = []
    for e in random_trace(7, 300, rate=400.0, poll_dt=0.004, burstiness=[0.5, 0.4, 0.1]):
        ev.append(e if e[0] == "push" else ("poll", e[1], int(g.integers(1, 12))))
    assert run_native(ev, 8, 0.03, 0)[0] == BO.simulate(ev, 8, 0.03, 0)


def test_native_queue_deadline_errors_and_threads():
    L = B.lib()
    q = B.Batcher(4, 0.25)
    assert q.deadline() == math.inf and q.poll(1e9) == []
    q.push(7, 3, 2, 10.0)
    q.push(8, 3, 2, 9.0)                     # stamp older than the previous push: raised, order kept
    assert q.deadline() == 10.25
    assert q.poll(10.2) == []
    assert q.poll(10.25) == [(7, 3, 2, 10.0), (8, 3, 2, 10.0)]
    for bad in [(1, 0, 0, 0.0), (1, -1, 5, 0.0), (1, 1, 1, float("nan"))]:
        with pytest.raises(B.VlaError):
            q.push(*bad)
    small = (B.vla_request * 2)()
    import ctypes as C
    n = C.c_int32()
    assert L.vla_batcher_poll(q.h, 0.0, small, 0, C.byref(n)) == -4           # nothing can be taken
    h = C.c_void_p()
    assert L.vla_batcher_create(0, 1.0, 0, C.byref(h)) == -2
    assert L.vla_batcher_create(4, -1.0, 0, C.byref(h)) == -2
    assert L.vla_batcher_create(4, float("inf"), 0, C.byref(h)) == -2
    capq = B.Batcher(4, 1.0, max_tokens=100)
    with pytest.raises(B.VlaError) as e:
        capq.push(1, 80, 30, 0.0)
    assert e.value.code == -4
    capq.close()
    # pushes from several threads while the worker polls: nothing lost, nothing duplicated, batches <= B
    got, lock = [], threading.Lock()

    def producer(base):
        for i in range(2000):
            q.push(base + i, 1, 1, 20.0)

    th = [threading.Thread(target=producer, args=(k * 10000,)) for k in range(4)]
    for t in th:
        t.start()
    while any(t.is_alive() for t in th) or len(q):
        b = q.poll(1e6)
        assert len(b) <= 4
        got += [r[0] for r in b]
    for t in th:
        t.join()
    assert sorted(got) == sorted(k * 10000 + i for k in range(4) for i in range(2000))
    for k in range(4):                       # per-producer order is preserved (FIFO)
        mine = [r for r in got if r // 10000 == k]
        assert mine == sorted(mine)
    q.close()
