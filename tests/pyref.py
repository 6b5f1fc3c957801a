"""Brute-force Python re-statement of the buffer policy for tiny inputs.

Written independently of oracle/rbo.c (Python integers, sets, lists and
dictionaries instead of C arrays) so that the two can be compared on small
cases.  It follows Algorithm 1 and the sampling rule of Sec. IV-C of the paper
with the same reading of the silent points (counter-based draws, ascending
mini-batch position, uniform eviction, class-major numbering of stored
samples).
"""

MASK32 = 0xFFFFFFFF
SELECT, EVICT, SAMPLE, COIN = 1, 2, 3, 4


def philox4x32_10(ctr, key):
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK32, p1 & MASK32, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK32, p0 & MASK32]
        k = [(k[0] + 0x9E3779B9) & MASK32, (k[1] + 0xBB67AE85) & MASK32]
    return c


def draw64(seed, step, purpose, index):
    w = philox4x32_10([index, purpose, step & MASK32, (step >> 32) & MASK32], [seed & MASK32, (seed >> 32) & MASK32])
    return w[0] | (w[1] << 32)


def bounded(seed, step, purpose, index, n):
    return (draw64(seed, step, purpose, index) * n) >> 64


def floyd(seed, step, purpose, n, m):
    chosen, order = set(), []
    for i in range(m):
        j = n - m + i
        t = bounded(seed, step, purpose, i, j + 1)
        x = j if t in chosen else t
        chosen.add(x)
        order.append(x)
    return order


class PyBuffer:
    def __init__(self, K, S, selection="exact", eviction="uniform"):
        self.K, self.S = K, S
        self.R = {k: [] for k in range(K)}     # class -> list of stored rows (bytes objects), index = slot
        self.bad_label = False
        self.selection, self.eviction = selection, eviction
        self.age = {k: [] for k in range(K)}   # fifo: arrival number of what each slot holds
        self.offered = {k: 0 for k in range(K)}

    def update(self, rows, labels, c, seed, step):
        b = len(labels)
        if self.selection == "bernoulli":
            chosen = [pos for pos in range(b) if bounded(seed, step, COIN, pos, b) < c]
        else:
            chosen = sorted(floyd(seed, step, SELECT, b, c))
        for pos in chosen:
            k = labels[pos]
            if not (0 <= k < self.K):
                self.bad_label = True
                continue
            sub = self.R[k]
            n = self.offered[k]
            self.offered[k] += 1
            if len(sub) < self.S:
                sub.append(rows[pos])
                self.age[k].append(n)
            elif self.eviction == "fifo":
                oldest = min(range(self.S), key=lambda s: self.age[k][s])
                sub[oldest] = rows[pos]
                self.age[k][oldest] = n
            elif self.eviction == "reservoir":
                j = bounded(seed, step, EVICT, pos, n + 1)
                if j < self.S:
                    sub[j] = rows[pos]
            else:
                sub[bounded(seed, step, EVICT, pos, self.S)] = rows[pos]

    def stored(self):
        """Every stored sample as (class, slot, row), class after class."""
        return [(k, s, row) for k in range(self.K) for s, row in enumerate(self.R[k])]

    def sample(self, r, seed, step):
        flat = self.stored()
        n = min(r, len(flat))
        return [flat[g] for g in floyd(seed, step, SAMPLE, len(flat), n)]
