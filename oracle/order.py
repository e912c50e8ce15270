"""Partition loading order and edge-bucket iteration order (oracle; test infrastructure).

Sec. 4 of the paper: buffer capacity 3, n > 3 partitions, one partition swapped
per buffer state, "column separation covering" (Alg. 1) and the bucket order
derived from it (Alg. 2).  Both printed listings are damaged; the steps below
follow the prose and the n = 6 worked example, and are the reading recorded in
the design notes:

Alg. 1
  * states {0,1,2}, then swap in 3..n-1 in id order, each time evicting the
    partition loaded two states earlier (column 0 gets covered);
  * when the current column is fully covered, move to the next column by
    swapping the column partition for its successor (if the successor is already
    resident the column simply advances); then, of the two other residents,
    evict the larger id if the new column still has an uncovered bucket beyond
    it, else the smaller id;
  * otherwise evict the resident that is neither the column partition nor the
    one loaded last (property (1) of Theorem 1);
  * load the non-resident id that newly covers the most partition pairs with
    the two that stay, scanning ids cyclically from max(buffer)+1, first best wins.

Alg. 2
  * per buffer state, first the not-yet-trained buckets that involve the
    partition evicted next (those pairing it with the partition loaded last come
    last of these), then - while the swap is in flight - the remaining untrained
    buckets of the state;
  * the last state trains everything still untrained.
"""

from __future__ import annotations

from typing import List, Tuple


def loading_order(n: int) -> List[Tuple[int, int, int]]:
    """Buffer states in order; each state lists its residents by buffer slot, so
    consecutive states differ in exactly one slot."""
    if n <= 3:
        return [tuple(range(n)) + (-1,) * (3 - n)]
    covered = [[False] * n for _ in range(n)]

    def mark(buf):
        for a in buf:
            for b in buf:
                covered[a][b] = True

    def done():
        return all(all(row) for row in covered)

    buf = [0, 1, 2]
    states = [tuple(buf)]
    mark(buf)
    for p in range(3, n):
        buf[buf.index(p - 2)] = p
        states.append(tuple(buf))
        mark(buf)

    col = 0
    last_loaded = n - 1
    while not done():
        if all(covered[col]):
            nxt = col + 1
            if nxt in buf:
                col = nxt
                continue
            buf[buf.index(col)] = nxt
            states.append(tuple(buf))
            mark(buf)
            col = nxt
            last_loaded = nxt
            if done():
                break
            others = sorted(x for x in buf if x != col)
            beyond_uncovered = any(not covered[col][x] for x in range(others[1] + 1, n))
            evict = others[1] if beyond_uncovered else others[0]
        else:
            evict = next(x for x in buf if x != col and x != last_loaded)
        stay = [x for x in buf if x != evict]
        begin = max(buf) + 1
        best, best_gain = -1, -1
        for t in range(n):
            cand = (begin + t) % n
            if cand in buf:
                continue
            gain = sum(1 for r in stay if not covered[r][cand])
            if gain > best_gain:
                best, best_gain = cand, gain
        buf[buf.index(evict)] = best
        last_loaded = best
        states.append(tuple(buf))
        mark(buf)
    return states


def iteration_order(states: List[Tuple[int, int, int]], n: int):
    """Bucket order per buffer state.

    Returns a list with one entry per state:
        (evict, load, before_swap, during_swap)
    evict/load: partition swapped out of / into the buffer to reach the next
    state (-1, -1 for the last state); before_swap: buckets to train before the
    swap may start (they involve `evict`); during_swap: buckets trained while
    the swap is in flight (they do not involve `evict`)."""
    trained = [[False] * n for _ in range(n)]
    plan = []
    loaded_last = -1
    for k, st in enumerate(states):
        res = [x for x in st if x >= 0]
        if k + 1 < len(states):
            nxt = states[k + 1]
            evict = next(x for x in st if x not in nxt)
            load = next(x for x in nxt if x not in st)
        else:
            evict, load = -1, -1
        before, during = [], []

        def take(a, b, dest):
            if not trained[a][b]:
                trained[a][b] = True
                dest.append((a, b))

        if evict >= 0:
            first = [x for x in res if x != loaded_last] + [x for x in res if x == loaded_last]
            for kx in first:
                take(evict, kx, before)
                if kx != evict:
                    take(kx, evict, before)
        for a in sorted(res):
            for b in sorted(res):
                if a != evict and b != evict:
                    take(a, b, during)
        plan.append((evict, load, before, during))
        loaded_last = load
    return plan
