"""BETA edge-bucket ordering and the partition-buffer simulator (oracle side; test infrastructure).

Sec. 4.1: an edge-bucket ordering is viewed as a sequence of partition buffers in which each
successive buffer differs by one swapped partition.  Alg. 3 builds the BETA buffer sequence, Alg. 4
turns a buffer sequence into an edge-bucket order (every pair the first time both partitions are in
the buffer, shuffled within a buffer), Alg. 2 replays an order through a buffer of c partitions that
evicts the partition used furthest in the future.  Eq. 2 is the lower bound on swaps, Eq. 3 the swap
count of BETA; filling the first buffer is not counted as swaps.

Reading of the shuffle (the paper only says "shuffle"): Fisher-Yates from the back with
j = mulhi64(x, k + 1), x = words (0, 1) of Philox4x32-10 with key = seed and counter
(k, buffer index, 0, 0x40000000).
"""
import math

from .philox import philox4x32_10, mulhi64


def beta_buffer_sequence(p, c):
    """Alg. 3.  Returns the list of buffers (each a list of c partition ids)."""
    assert 2 <= c <= p
    seq = []
    current = list(range(c))
    on_disk = list(range(c, p))
    seq.append(list(current))
    while on_disk:
        # keep the leading c-1 partitions, cycle every partition on disk through the last slot
        for i in range(len(on_disk)):
            current[-1], on_disk[i] = on_disk[i], current[-1]
            seq.append(list(current))
        # the leading partitions have met everybody: replace them by fresh ones from disk
        n = 0
        for i in range(c - 1):
            if i >= len(on_disk):
                break
            n += 1
            current[i] = on_disk[i]
            seq.append(list(current))
        on_disk = on_disk[n:]
    return seq


def shuffle_in_place(items, seed, buffer_index):
    for k in range(len(items) - 1, 0, -1):
        o = philox4x32_10((k, buffer_index, 0, 0x40000000), (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
        j = mulhi64(o[0] | (o[1] << 32), k + 1)
        items[k], items[j] = items[j], items[k]


def edge_bucket_order(buffers, p, seed=None):
    """Alg. 4.  Returns the list of (i, j) edge buckets; seed=None keeps the generation order."""
    seen = [[False] * p for _ in range(p)]
    order = []
    for b, buf in enumerate(buffers):
        new = []
        for i in buf:
            for j in buf:
                if not seen[i][j]:
                    seen[i][j] = True
                    new.append((i, j))
        if seed is not None:
            shuffle_in_place(new, seed, b)
        order.extend(new)
    return order


def simulate_buffer(order, c):
    """Alg. 2 without the training: returns the number of partition loads; swaps = loads - c once the
    buffer has been filled (the first c loads fill it)."""
    n = len(order)
    buf = []
    loads = 0
    for k, (i, j) in enumerate(order):
        for x in (i, j):
            if x in buf:
                continue
            if len(buf) == c:
                # evict the partition whose next use is furthest in the future (never one needed now)
                far, victim = -1, None
                for y in buf:
                    if y == i or y == j:
                        continue
                    nxt = n
                    for t in range(k, n):
                        if y == order[t][0] or y == order[t][1]:
                            nxt = t
                            break
                    if nxt > far:
                        far, victim = nxt, y
                buf.remove(victim)
            buf.append(x)
            loads += 1
    return loads


def swap_lower_bound(p, c):
    """Eq. 2."""
    return math.ceil((p * (p - 1) // 2 - c * (c - 1) // 2) / (c - 1))


def beta_swap_count(p, c):
    """Eq. 3."""
    x = (p - c) // (c - 1)
    twice = 2 * (p - c) + (x + 1) * (2 * (p - c) - x * (c - 1))
    assert twice % 2 == 0
    return twice // 2
