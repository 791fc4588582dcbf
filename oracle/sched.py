"""CPU oracle of the host-side scheduler pieces (section "SLO-Aware Scheduler").

TEST INFRASTRUCTURE ONLY (imported by tests; never by the product path; shares no code with it).

* slack score (section "SLO-based Scheduling Algorithm"):  Slack_i = (DDL_i - C_i - P_i) / SA_i  with DDL_i the
  request's SLO budget, C_i the time since it arrived, P_i the predicted time of its remaining steps and SA_i its
  standalone latency.  Lower = more urgent.
* latency model in place of the paper's MLP (section "Mixed-Resolution Throughput Analyzer": inputs are the number of
  tasks per resolution, the number of resolutions in flight and the total patch number; the MLP itself needs the
  authors' measurements).  Here: per-step batch latency = w0 + w1 * patches + w2 * distinct resolutions
  + w3 * 1e-6 * sum_i tokens_i^2 (the attention term, which is what the per-resolution task counts drive), fitted by
  ordinary least squares on measured (batch, latency) samples.
* the scheduling loop (the paper's Algorithm "schedule algorithm"), in its order: take the least-slack waiting task and
  the least-slack active task; predict the latency of the batch with the candidate; discard the candidate if it cannot
  meet its deadline even so; if its slack is relaxed, switch to the throughput mode and take instead the waiting task
  that maximises batch tokens per predicted millisecond; stop when the least-slack active task would miss its
  deadline with the candidate on board, else admit and repeat.

Readings (the listing leaves the helper functions open):
  time_out(task, latency)   : now + steps_left * latency > arrival + DDL
  P_i                       : steps_left_i * (latency predicted for the batch under consideration)
  switch_mode               : slack(candidate) > relaxed_slack (a parameter)
  update_task               : among waiting tasks that do not time out in the batch they would join, the one with the
                              largest (tokens of active + task) / latency(active + task); ties: first in queue order
  least slack               : ties go to the first in queue order
  an admitted task counts as active for the following iterations; a discarded one leaves the waiting queue
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np


@dataclass
class Task:
    id: int
    H: int
    W: int
    steps_left: int
    arrival: float       # ms
    ddl: float           # SLO budget from arrival, ms
    standalone: float    # SA: latency of the request run alone, ms


def features(batch: Sequence[Task], ph: int, pw: int) -> Tuple[float, float, float]:
    patches = sum((t.H // ph) * (t.W // pw) for t in batch)
    resolutions = len({(t.H, t.W) for t in batch})
    attn = 1e-6 * sum(float(t.H * t.W) ** 2 for t in batch)
    return float(patches), float(resolutions), attn


def predict(w: Sequence[float], batch: Sequence[Task], ph: int, pw: int) -> float:
    p, r, a = features(batch, ph, pw)
    return w[0] + w[1] * p + w[2] * r + w[3] * a


def fit(X: np.ndarray, y: np.ndarray) -> np.ndarray:
    """Least squares of y ~ [1, X] (X [m][3]); returns w[4]."""
    A = np.concatenate([np.ones((X.shape[0], 1)), np.asarray(X, dtype=np.float64)], axis=1)
    return np.linalg.lstsq(A, np.asarray(y, dtype=np.float64), rcond=None)[0]


def slack(t: Task, now: float, latency: float) -> float:
    return (t.ddl - (now - t.arrival) - t.steps_left * latency) / t.standalone


def time_out(t: Task, now: float, latency: float) -> bool:
    return now + t.steps_left * latency > t.arrival + t.ddl


def schedule(wait: Sequence[Task], active: Sequence[Task], now: float, w: Sequence[float], ph: int, pw: int,
             relaxed_slack: float) -> Tuple[List[int], List[int]]:
    """Returns (admitted, discarded): indices into `wait`, in the order decided."""
    waiting = list(range(len(wait)))
    act: List[Task] = list(active)
    admitted: List[int] = []
    discarded: List[int] = []
    while waiting:
        lat_now = predict(w, act, ph, pw) if act else 0.0
        # least-slack waiting task, scored with the latency of the batch it would join
        best, best_s = None, None
        for i in waiting:
            s = slack(wait[i], now, predict(w, act + [wait[i]], ph, pw))
            if best is None or s < best_s:
                best, best_s = i, s
        cur = best
        act_task = None
        if act:
            act_task = min(range(len(act)), key=lambda k: (slack(act[k], now, lat_now), k))
        pred = predict(w, act + [wait[cur]], ph, pw)
        if time_out(wait[cur], now, pred):                       # cannot meet its deadline even if run now
            discarded.append(cur)
            waiting.remove(cur)
            continue
        if best_s > relaxed_slack:                               # throughput mode
            tok_act = sum(t.H * t.W for t in act)
            top, top_v = None, None
            for i in waiting:
                lat_i = predict(w, act + [wait[i]], ph, pw)
                if time_out(wait[i], now, lat_i):
                    continue
                v = (tok_act + wait[i].H * wait[i].W) / lat_i
                if top is None or v > top_v:
                    top, top_v = i, v
            cur = top                                            # never None: the first candidate itself qualifies
            pred = predict(w, act + [wait[cur]], ph, pw)
        if act_task is not None and time_out(act[act_task], now, pred):
            break                                                # the most urgent running task would miss its deadline
        admitted.append(cur)
        waiting.remove(cur)
        act.append(wait[cur])
    return admitted, discarded
