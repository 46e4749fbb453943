"""Plain-Python oracle of the length-aware tile scheduler's work list.  TEST INFRASTRUCTURE ONLY.

The paper motivates its design with the imbalance that mixed long and short samples cause (Section
2.2, Section 4.1.1) and picks its attention algorithm for its work partitioning on long inputs
(Section 6, "Efficient Operators"); it gives no scheduling algorithm.  The reading taken by the
library: a packed batch is cut into row tiles of `tile_rows` rows per sample, a tile's cost is the
number of partner tiles of `partner_rows` rows it has to visit, and tiles are handed out heaviest
first.  This file states which tiles exist and what each costs, straight from the attention mask:

    full            every row tile of a sample meets the whole sample
    causal_query    the tile holds queries; it meets the keys j <= i of its rows i
    causal_key      the tile holds keys; it meets the queries i >= j of its rows j

The order of tiles of equal cost is left open (the device list may take any).
"""

MODES = ("full", "causal_query", "causal_key")


def work_items(cu_seqlens, tile_rows, partner_rows, mode):
    """List of (first_row, sample_begin, sample_end, tile_index, cost), in sample order."""
    assert mode in MODES
    items = []
    for s in range(len(cu_seqlens) - 1):
        begin, end = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        L = end - begin
        tiles = -(-L // tile_rows)
        for t in range(tiles):
            if mode == "full":
                rows_met = L
            elif mode == "causal_query":          # keys 0 .. last query row of the tile
                rows_met = min(L, (t + 1) * tile_rows)
            else:                                 # queries first key row of the tile .. L-1
                rows_met = L - t * tile_rows
            cost = -(-rows_met // partner_rows)
            items.append((begin + t * tile_rows, begin, end, t, cost))
    return items


def cost_by_brute_force(L, t, tile_rows, partner_rows, mode):
    """The same cost counted from the mask itself: partner tiles that hold at least one allowed pair."""
    rows = range(t * tile_rows, min(L, (t + 1) * tile_rows))
    met = set()
    for a in rows:
        for b in range(L):
            if mode == "full":
                ok = True
            elif mode == "causal_query":   # a is the query, b the key
                ok = b <= a
            else:                          # a is the key, b the query
                ok = b >= a
            if ok:
                met.add(b // partner_rows)
    return len(met)
