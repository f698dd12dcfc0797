"""Plain definition of the level packing of a serial event stream (test infrastructure).

A batch is a window of consecutive events of the serial stream.  Inside a batch,
an event's level is one more than the highest level of any earlier event of the batch
that shares a worker with it (0 if there is none).  Events of one level therefore touch
pairwise disjoint workers (a matching plus singletons), and every worker meets its events
in increasing level, i.e. in serial order.  Inside a level events keep their serial order.
"""


def pack(kind, wi, wj, batch_size):
    """Returns a list of batches; a batch is a list of levels; a level is a list of serial indices."""
    batches = []
    m = len(kind)
    for lo in range(0, m, batch_size):
        hi = min(m, lo + batch_size)
        last = {}
        levels = []
        for e in range(lo, hi):
            workers = [int(wi[e])] if kind[e] == 0 else [int(wi[e]), int(wj[e])]
            lev = 1 + max((last.get(w, -1) for w in workers))
            for w in workers:
                last[w] = lev
            while len(levels) <= lev:
                levels.append([])
            levels[lev].append(e)
        batches.append(levels)
    return batches
