"""Plain-Python oracle of the length-balanced partitioner.  TEST INFRASTRUCTURE ONLY.

The paper balances encoder workloads by reordering the samples of a group of ranks "using the Karp
algorithm" (Section 5.1, decentralized grouped reordering) and gives no further detail.  The reading
taken here: the samples' costs are split into `bins` subsets (one per rank) so that the largest
subset cost is small, with the Karmarkar-Karp largest differencing method in its k-way form, and
greedy longest-processing-time-first list scheduling as the comparison.  Everything below is the
textbook statement of the two methods written out with lists and full sorts: slow, small inputs only.

Cost of a sample of length L: lin * L + quad * L * L (attention is the quadratic term).

Conventions shared with the library (they fix the result where the methods leave freedom):
  * ties between samples of equal cost go to the lower index; ties between bins to the lower bin;
  * a partial solution of the differencing method is a list of `bins` slots [cost, members], kept
    sorted by cost descending with a stable sort; its spread is first cost - last cost;
  * each round merges the two partial solutions of largest spread (ties: the one created earlier
    first), slot j of the first with slot bins-1-j of the second;
  * equal_counts: the start is not one sample per partial solution but `bins` consecutive samples
    of the cost-sorted order, one per slot (the balanced variant: bin sizes then differ by <= 1);
  * the bins are the slots of the last partial solution: bin 0 is the most expensive one.
"""


def costs(lengths, lin, quad):
    return [float(lin) * float(L) + float(quad) * float(L) * float(L) for L in lengths]


def karmarkar_karp(lengths, bins, lin=0.0, quad=1.0, equal_counts=False):
    """Returns bin_of[i] for every sample."""
    c = costs(lengths, lin, quad)
    n = len(c)
    order = sorted(range(n), key=lambda i: (-c[i], i))
    sols = []  # [creation number, slots]
    if equal_counts:
        for g in range(0, n, bins):
            slots = [[c[i], [i]] for i in order[g:g + bins]]
            slots += [[0.0, []] for _ in range(bins - len(slots))]
            sols.append([len(sols), slots])
    else:
        for i in order:
            sols.append([len(sols), [[c[i], [i]]] + [[0.0, []] for _ in range(bins - 1)]])
    created = len(sols)
    while len(sols) > 1:
        sols.sort(key=lambda s: (-(s[1][0][0] - s[1][-1][0]), s[0]))
        a, b = sols[0][1], sols[1][1]
        merged = [[a[j][0] + b[bins - 1 - j][0], a[j][1] + b[bins - 1 - j][1]] for j in range(bins)]
        merged.sort(key=lambda slot: -slot[0])  # stable
        sols = sols[2:] + [[created, merged]]
        created += 1
    bin_of = [0] * n
    if sols:
        for b, (_, members) in enumerate(sols[0][1]):
            for i in members:
                bin_of[i] = b
    return bin_of


def lpt(lengths, bins, lin=0.0, quad=1.0, equal_counts=False):
    """Greedy: samples by decreasing cost, each to the currently cheapest bin (that still has room)."""
    c = costs(lengths, lin, quad)
    n = len(c)
    lo, extra = n // bins, n % bins  # equal_counts: `extra` bins hold lo + 1 samples, the others lo
    total = [0.0] * bins
    count = [0] * bins
    bin_of = [0] * n

    def has_room(b):
        if not equal_counts:
            return True
        full_bins = sum(1 for x in count if x == lo + 1)
        return count[b] < lo or (count[b] == lo and full_bins < extra)

    for i in sorted(range(n), key=lambda i: (-c[i], i)):
        b = min((b for b in range(bins) if has_room(b)), key=lambda b: (total[b], b))
        bin_of[i] = b
        total[b] += c[i]
        count[b] += 1
    return bin_of


def bin_costs(lengths, bin_of, bins, lin=0.0, quad=1.0):
    c = costs(lengths, lin, quad)
    out = [0.0] * bins
    for i, b in enumerate(bin_of):
        out[b] += c[i]
    return out


def optimum_max_cost(lengths, bins, lin=0.0, quad=1.0):
    """Smallest possible largest-bin cost, by trying every assignment (tiny inputs only)."""
    c = costs(lengths, lin, quad)
    best = [float("inf")]
    total = [0.0] * bins

    def rec(i):
        if i == len(c):
            best[0] = min(best[0], max(total))
            return
        seen_empty = False
        for b in range(bins):
            if total[b] == 0.0:
                if seen_empty:
                    continue  # bins are interchangeable: one empty bin is enough to try
                seen_empty = True
            total[b] += c[i]
            if max(total) < best[0]:
                rec(i + 1)
            total[b] -= c[i]
    rec(0)
    return best[0]
