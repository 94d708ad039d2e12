"""Oracle of the Inference Worker's dynamic-window batching rule (Section 3.2, Eq. 1).

TEST INFRASTRUCTURE ONLY: imported by tests/; the product path (the native queue in the HIP library)
shares no code with it.

The worker keeps a FIFO request queue Q.  Whenever it looks at the queue (a "poll" at time t_now) a batched
forward pass is triggered iff
        |Q| >= B   or   t_now - t_first >= T_max,
where t_first is the arrival time of the oldest queued request.  Readings where the paper is silent: an empty
queue never triggers; a triggered batch takes the oldest requests, at most B of them and, if a token capacity
is given, only while the packed prefix tokens fit (always at least one request); the rest keep their place and
their own arrival times, so the rule can fire again at once.
"""
from typing import List, Sequence, Tuple


def trigger(q_len: int, B: int, t_now: float, t_first: float, T_max: float) -> bool:
    """Eq. 1 for a non-empty queue; False for an empty one."""
    if q_len <= 0:
        return False
    return q_len >= B or (t_now - t_first) >= T_max


def simulate(events: Sequence[Tuple], B: int, T_max: float, max_tokens: int = 0) -> List[Tuple[float, List[int]]]:
    """events, in the order the worker sees them:
         ("push", t_arrival, request_id, n_tokens)   a request joins the back of Q
         ("poll", t_now[, cap])                      the worker evaluates Eq. 1 once; cap (default B) is the most
                                                     requests it can take at this moment
    Returns one (t_now, [request ids]) per poll that triggered."""
    Q: List[Tuple[float, int, int]] = []
    out = []
    for ev in events:
        if ev[0] == "push":
            _, t, rid, n_tok = ev
            Q.append((t, rid, n_tok))
        else:
            t_now = ev[1]
            if not trigger(len(Q), B, t_now, Q[0][0] if Q else 0.0, T_max):
                continue
            batch, tokens = [], 0
            most = min(B, ev[2]) if len(ev) > 2 else B
            while Q and len(batch) < most:
                if max_tokens and batch and tokens + Q[0][2] > max_tokens:
                    break
                t, rid, n_tok = Q.pop(0)
                batch.append(rid)
                tokens += n_tok
            out.append((t_now, batch))
    return out


def deadline(Q_arrivals: Sequence[float], T_max: float) -> float:
    """Earliest time at which the waiting-time clause alone fires: t_first + T_max (inf if Q is empty)."""
    return (Q_arrivals[0] + T_max) if len(Q_arrivals) else float("inf")
