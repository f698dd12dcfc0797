"""The paper's practical event source (test infrastructure): gradient steps back to back, a Poisson
number of p2p averagings per gradient step, partners found first-in-first-out among available
neighbours (section "Practical implementation of the dynamic"; appendix "Uniform neighbor selection
check").  Plain Python, one event at a time.

Reading used (the paper describes the mechanism in prose only):
  * worker i finishes gradient steps back to back; the k-th step lasts (1 / rate_i) * (1 + jitter * (2u - 1)),
    u uniform in [0, 1); its completion at time t is the gradient event (t, i);
  * at each completion the worker draws K ~ Poisson(comm_per_grad) and adds K to the averagings it still
    has to do;
  * a worker is AVAILABLE when it is not inside an averaging and still has averagings to do; when it
    becomes available it joins the tail of one global queue;
  * whenever the queue changes, the coordinator scans it from the head and pairs the first worker with
    the first later worker that is its neighbour in the graph, as long as such pairs exist; a pairing at
    time t is the gossip event (t, i, j), costs each partner one of its pending averagings and keeps both
    busy until t + comm_time;
  * simultaneous completions are handled in order (time, communication-end before gradient-end, worker id);
  * normalize=True (the same section: a running average of the duration of the previous gradient steps
    normalises time, so that a gradient step takes one unit as the analysis assumes): events are stamped with
    the normalised time T, which advances by (real time elapsed) / (average duration of all gradient steps
    completed so far, by any worker); before the first completion the average is the mean of 1 / rate_i.  A
    step's duration enters the average after the events of its own completion are stamped.  Durations and
    communication times stay in real time; only the stamps change.
  * normalize="worker": the same sentence read per worker.  Every worker normalises its own clock by the running
    average of the durations of its OWN previous gradient steps (before its first completion: 1 / rate_i).  Events
    keep their real-time stamps, which order them; what changes is how much time elapses for the mixing of worker
    i between two of its events: (real time elapsed) / (worker i's average).  The stream carries this as the field
    `speed` of a gradient event: the speed of that worker's clock from the event on, 1 / (average duration of the
    worker's steps completed so far, the one just finished included), rounded to fp32, the precision in which the
    engine receives it.  As above, a step's duration counts only after the events of its own completion.  The
    initial speeds are the rates rate_i (core.State.rate has to be set to them).

Random numbers: Philox4x32-10, key = (seed_lo, seed_hi), counter = (draw_lo, draw_hi, worker, tag) with
tag 0x0A2C1D21 for step durations and 0x0A2C1D22 for the Poisson counts; a uniform is the 53-bit value
built from words 0 and 1.  The Poisson count multiplies uniforms until the product drops to exp(-mean) or
below (Knuth).
"""
import heapq
import math

import numpy as np

from . import core

TAG_DURATION = 0x0A2C1D21
TAG_POISSON = 0x0A2C1D22


class _Uniforms:
    def __init__(self, seed, worker, tag):
        self.key = [seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF]
        self.worker, self.tag, self.k = worker, tag, 0

    def next(self):
        w = core.philox4x32_10([self.k & 0xFFFFFFFF, self.k >> 32, self.worker, self.tag], self.key)
        self.k += 1
        return ((int(w[0]) << 21) | (int(w[1]) >> 11)) * 2.0 ** -53


def _poisson(stream, mean):
    limit = math.exp(-mean)
    k, p = 0, 1.0
    while True:
        k += 1
        p *= stream.next()
        if not p > limit:
            return k - 1


def generate(n, edges, node_rate, comm_per_grad, comm_time, jitter, seed, n_events, normalize=False):
    """Returns core.Events (clock = worker for gradient events, n + edge index for gossip events; speed: see
    normalize="worker", else None)."""
    per_worker = normalize == "worker"
    if per_worker:
        normalize = False
    edge_index = {}
    for e, (a, b) in enumerate(edges):
        edge_index[(a, b)] = e
        edge_index[(b, a)] = e
    dur = [_Uniforms(seed, i, TAG_DURATION) for i in range(n)]
    cnt = [_Uniforms(seed, i, TAG_POISSON) for i in range(n)]
    todo = [0] * n
    busy = [False] * n
    queue = []                                   # available workers, oldest first
    heap = []                                    # (time, kind: 0 communication end / 1 gradient end, worker)
    running = [0.0] * n                          # duration of the gradient step each worker is in
    for i in range(n):
        if node_rate[i] > 0:
            running[i] = (1.0 / node_rate[i]) * (1.0 + jitter * (2.0 * dur[i].next() - 1.0))
            heapq.heappush(heap, (running[i], 1, i))
    out_t, out_kind, out_i, out_j, out_clock, out_speed = [], [], [], [], [], []
    own_sum, own_n = [0.0] * n, [0] * n          # per worker: durations of its completed gradient steps
    active = [1.0 / node_rate[i] for i in range(n) if node_rate[i] > 0]
    unit = sum(active) / len(active) if active else 1.0      # average gradient-step duration so far
    dur_sum, dur_n = 0.0, 0
    t_norm, real_last = 0.0, 0.0

    def join(i):
        if not busy[i] and todo[i] > 0 and i not in queue:
            queue.append(i)

    def match(t):
        while True:
            found = None
            for pa in range(len(queue)):
                for pb in range(pa + 1, len(queue)):
                    if (queue[pa], queue[pb]) in edge_index:
                        found = (pa, pb)
                        break
                if found:
                    break
            if not found or len(out_t) >= n_events:
                return
            a, b = queue[found[0]], queue[found[1]]
            del queue[found[1]]
            del queue[found[0]]
            e = edge_index[(a, b)]
            out_t.append(stamp(t)); out_kind.append(1); out_i.append(edges[e][0]); out_j.append(edges[e][1])
            out_clock.append(n + e)
            out_speed.append(0.0)
            for w in (a, b):
                todo[w] -= 1
                busy[w] = True
                heapq.heappush(heap, (t + comm_time, 0, w))

    def stamp(t):
        return t_norm if normalize else t

    while heap and len(out_t) < n_events:
        t, kind, i = heapq.heappop(heap)
        t_norm += (t - real_last) / unit
        real_last = t
        if kind == 0:
            busy[i] = False
        else:
            out_t.append(stamp(t)); out_kind.append(0); out_i.append(i); out_j.append(-1); out_clock.append(i)
            todo[i] += _poisson(cnt[i], comm_per_grad)
            finished = running[i]
            own_sum[i] += finished
            own_n[i] += 1
            out_speed.append(float(np.float32(1.0 / (own_sum[i] / own_n[i]))))
            running[i] = (1.0 / node_rate[i]) * (1.0 + jitter * (2.0 * dur[i].next() - 1.0))
            heapq.heappush(heap, (t + running[i], 1, i))
        join(i)
        match(t)
        if kind == 1:                            # the finished step counts from the next interval on
            dur_sum += finished
            dur_n += 1
            unit = dur_sum / dur_n
    return core.Events(np.array(out_t), np.array(out_kind, np.int32), np.array(out_i, np.int32),
                       np.array(out_j, np.int32), np.array(out_clock, np.int32),
                       np.array(out_speed) if per_worker else None)
