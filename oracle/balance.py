"""Oracle for token-balanced dispatch.  TEST INFRASTRUCTURE ONLY (same rules as the rest of this package).

The paper balances work across data-parallel groups by treating it as one-dimensional bin packing solved with
the Karmarkar-Karp algorithm (Sec. 4.4): equal sample counts per group and a small spread of token totals for
data parallelism, the count constraint relaxed for pipeline parallelism.  It gives no further detail, so this
follows the published algorithm (Karmarkar and Karp 1982, the largest differencing method, in its k-way form,
and its count-balanced variant that starts from groups of k consecutive items of the sorted list), with every
choice the publications leave open fixed as follows so that the result is unique:

  partial solution   k sets, kept in order of decreasing sum (ties: the set whose smallest item index is
                     smaller comes first; an empty set counts as index +infinity); spread = largest - smallest
  start, free        one partial solution per item i, sets ({i}, {}, ..., {}), created in input order
  start, equal count items sorted by decreasing weight (ties: smaller index first), padded with zero-weight
                     dummies to a multiple of k; one partial solution per k consecutive items, one item per set,
                     created in that order
  step               take the two partial solutions with the largest spread (ties: created earlier first), A
                     before B; merge set j of A with set k-1-j of B for every j; the result is created now
  end                one partial solution is left; its sets, in order, are parts 0..k-1

Plain Python, lists and a heap; nothing is shared with the C++ implementation.
"""
import heapq


def partition(weights, k, equal_count=False):
    """Returns part[i] in [0, k) for every item."""
    w = [int(x) for x in weights]
    n = len(w)
    if k < 1 or any(x < 0 for x in w):
        raise ValueError("k >= 1 and weights >= 0")
    INF = float("inf")

    def ordered(sets):  # sets: list of (sum, min_index, items)
        return sorted(sets, key=lambda s: (-s[0], s[1]))

    sols = []           # heap of (-spread, created, sets)
    created = 0
    if not equal_count:
        for i in range(n):
            sets = [(w[i], i, [i])] + [(0, INF, []) for _ in range(k - 1)]
            heapq.heappush(sols, (-(w[i] - (0 if k > 1 else w[i])), created, sets))
            created += 1
    else:
        order = sorted(range(n), key=lambda i: (-w[i], i))
        while len(order) % k:
            order.append(None)   # dummy
        for t in range(0, len(order), k):
            sets = []
            for i in order[t:t + k]:
                sets.append((0, INF, []) if i is None else (w[i], i, [i]))
            sets = ordered(sets)
            heapq.heappush(sols, (-(sets[0][0] - sets[-1][0]), created, sets))
            created += 1
    if not sols:
        return []
    while len(sols) > 1:
        _, _, a = heapq.heappop(sols)
        _, _, b = heapq.heappop(sols)
        merged = []
        for j in range(k):
            x, y = a[j], b[k - 1 - j]
            merged.append((x[0] + y[0], min(x[1], y[1]), x[2] + y[2]))
        merged = ordered(merged)
        heapq.heappush(sols, (-(merged[0][0] - merged[-1][0]), created, merged))
        created += 1
    part = [0] * n
    for p, s in enumerate(sols[0][2]):
        for i in s[2]:
            part[i] = p
    return part
