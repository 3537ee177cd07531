"""Algorithm 1 (rank -> precision class) and Algorithm 2 (tiered placement with
LRU promotion) of HA-RAG, as plain Python for small inputs.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Readings taken where the listings are silent or inconsistent:
  * a threshold times the chunk count is floored; thresholds are given in parts
    per million so that the product is an exact integer division;
  * equal access frequencies are ordered by ascending chunk id;
  * Algorithm 2 step 1 pairs tau_PIN with PIN_LIST and tau_PAGE with PAGE_LIST
    (the printed line swaps the two symbols), and ranks run 0..N-1;
  * a queue with a capacity evicts its least recently used member, the pinned
    queue included; `get` refreshes recency;
  * tiers are inclusive: promoting a chunk leaves the copy in the slower tier.
"""
from collections import OrderedDict

PPM = 1_000_000


def rank_order(af):
    """Algorithm 1 step 1: chunk ids sorted by access frequency, descending."""
    return sorted(range(len(af)), key=lambda i: (-int(af[i]), i))


def ranks(af):
    order = rank_order(af)
    r = [0] * len(af)
    for pos, cid in enumerate(order):
        r[cid] = pos
    return r


def split_points(n, taus_ppm):
    """Algorithm 1 step 2 / Algorithm 2 step 1: idx_k = floor(tau_k * n) + idx_{k-1}."""
    idx, acc = [], 0
    for t in taus_ppm:
        acc = min(n, acc + (int(t) * n) // PPM)
        idx.append(acc)
    return idx


def classes_by_rank(af, taus_ppm):
    """Class 0 = hottest ... len(taus) = coldest, per chunk id (Algorithm 1)."""
    order = rank_order(af)
    idx = split_points(len(af), taus_ppm)
    out = [0] * len(af)
    for pos, cid in enumerate(order):
        out[cid] = sum(1 for b in idx if pos >= b)
    return out


class _LRU:
    def __init__(self, cap):
        self.cap = cap  # None = unbounded
        self.d = OrderedDict()

    def __contains__(self, c):
        return c in self.d

    def get(self, c):
        self.d.move_to_end(c)

    def put(self, c):
        """Insert as most recent; returns the evicted id or None."""
        if c in self.d:
            self.d.move_to_end(c)
            return None
        ev = None
        if self.cap is not None and len(self.d) >= self.cap:
            if self.cap == 0:
                return c  # nothing fits: the chunk itself is not kept
            ev, _ = self.d.popitem(last=False)
        self.d[c] = True
        return ev

    def members(self):
        return list(self.d.keys())  # least recent first


class TierSim:
    """Algorithm 2 step 2 over a stream of accesses.

    rank[c]    0 = hottest (from Algorithm 1's sort)
    taus_ppm   (tau_GPU, tau_PIN, tau_PAGE)
    caps       (cap_GPU, cap_PIN, cap_PAGE); None = unbounded
    Chunks start on disk unless seeded with `seed(tier, ids)`.
    """

    GPU, PIN, PAGE, DISK = 0, 1, 2, 3

    def __init__(self, rank, taus_ppm, caps):
        self.rank = list(rank)
        n = len(rank)
        i1, i2, i3 = split_points(n, taus_ppm)
        self.bounds = (i1, i2, i3)
        self.q = [_LRU(caps[0]), _LRU(caps[1]), _LRU(caps[2])]

    def list_of(self, c):
        r = self.rank[c]
        i1, i2, i3 = self.bounds
        return self.GPU if r < i1 else self.PIN if r < i2 else self.PAGE if r < i3 else self.DISK

    def seed(self, tier, ids):
        for c in ids:
            self.q[tier].put(c)

    def access(self, c, floor=None):
        """Returns (tier the chunk was found in, [(tier placed into, evicted id or None)]).
        floor (an addition to the algorithm, for consumers that read chunks in place): no chunk
        is left in a tier slower than `floor`; its rank's list then counts as that tier."""
        placed = []
        want = self.list_of(c)
        if floor is not None and want > floor:
            want = floor
        if c in self.q[self.GPU]:
            self.q[self.GPU].get(c)
            return self.GPU, placed
        if c in self.q[self.PIN]:
            self.q[self.PIN].get(c)
            if want == self.GPU:
                placed.append((self.GPU, self.q[self.GPU].put(c)))
            return self.PIN, placed
        if c in self.q[self.PAGE]:
            self.q[self.PAGE].get(c)
            if want == self.GPU:
                placed.append((self.GPU, self.q[self.GPU].put(c)))
            if want == self.PIN:
                placed.append((self.PIN, self.q[self.PIN].put(c)))
            return self.PAGE, placed
        if want == self.GPU:
            placed.append((self.GPU, self.q[self.GPU].put(c)))
        if want == self.PIN:
            placed.append((self.PIN, self.q[self.PIN].put(c)))
        if want == self.PAGE:
            placed.append((self.PAGE, self.q[self.PAGE].put(c)))
        return self.DISK, placed

    def resident(self, tier):
        return self.q[tier].members()
