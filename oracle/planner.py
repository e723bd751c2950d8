"""Parallelism planning of the Jupiter paper (Sec. IV-B) -- TEST INFRASTRUCTURE, not a product path.

A plain statement of the two dynamic programs and of the latency estimate, next to exhaustive
enumerations of the same optimisation problems.  Only tests may import this module; it shares no code
with the library under test.

* Layer partition (Sec. IV-B.1, Eq. 1).  L layers, an ordered list of devices; stage n is a contiguous
  run of layers on device n; every device gets at least one layer.  T(i..j, n) is the sum of the
  profiled per-layer times of device n over layers i..j, +inf when the memory of those layers exceeds
  the device's budget.  A(1..y, D_n) = min over l of max(A(1..l, D_{n-1}), T(l+1..y, n)).
* Sequence partition (Sec. IV-B.2, Eq. 2 and 3).  W(1..y, k) = min over l of
  max(W(1..l, k-1), T*(y-l, l)), T*(x, l) = q(x, l) when x >= b, else +inf; W(1..y, 1) = T*(y, 0).
* Choice of k (Eq. 4).  Latency = sum of the sub-sequences' latencies h_i = q(|s_i|, tokens before s_i)
  plus (|D| - 1) times the slowest one.
* q(x, y) between profiled points (Sec. IV-B.2: results are approximated through interpolation):
  bilinear on the grid; above the largest profiled x and above the largest profiled y the outermost
  segment is continued linearly; below the smallest profiled x the latency of that smallest x is used
  (a shorter chunk is not faster once the accelerator is under-utilised), and below the smallest profiled
  y that of the smallest y (the paper interpolates, it does not extrapolate: a segment continued downwards
  can reach zero or below, and Eq. 2-4 mean nothing for a latency that is not positive).  For the same
  reason a continued value never falls below the smallest profiled latency.

Layers and tokens are numbered from 1 as in the paper; Python lists are 0-based, so layer i is t[i-1].
"""
import itertools
import math
from functools import lru_cache

INF = math.inf


# ---- q(x, y) from a profiled table ------------------------------------------------------------------
def _segment(grid, v, clamp_low):
    """Index i and weight w such that the value at v is (1-w)*f[i] + w*f[i+1]."""
    n = len(grid)
    if n == 1:
        return 0, 0.0
    if v <= grid[0]:
        if clamp_low:
            return 0, 0.0
        i = 0
    elif v >= grid[-1]:
        i = n - 2
    else:
        i = max(j for j in range(n - 1) if grid[j] <= v)
    return i, (v - grid[i]) / (grid[i + 1] - grid[i])


def interp_q(xs, ys, table, x, y):
    """table[i][j] = profiled latency of a chunk of xs[i] tokens behind ys[j] cached ones."""
    i, wx = _segment(xs, x, clamp_low=True)
    j, wy = _segment(ys, y, clamp_low=True)
    i2 = min(i + 1, len(xs) - 1)
    j2 = min(j + 1, len(ys) - 1)
    lo = (1.0 - wy) * table[i][j] + wy * table[i][j2]
    hi = (1.0 - wy) * table[i2][j] + wy * table[i2][j2]
    return max((1.0 - wx) * lo + wx * hi, min(min(row) for row in table))


# ---- Eq. 1: layers onto devices ------------------------------------------------------------------------
def stage_time(t, mem, budget, dev, i, j):
    """T(i..j, dev): layers i..j (1-based, inclusive) on device dev (0-based)."""
    if sum(mem[i - 1:j]) > budget[dev]:
        return INF
    return sum(t[dev][i - 1:j])


def layer_partition_dp(t, mem, budget):
    """Returns (A(1..L, D), last layer of every stage) following Eq. 1; ties: the smallest cut l."""
    n_dev, L = len(t), len(mem)

    @lru_cache(maxsize=None)
    def A(y, n):
        if n == 1:
            return stage_time(t, mem, budget, 0, 1, y), (y,)
        best, cuts = INF, None
        for l in range(n - 1, y):  # the first n-1 devices need at least one layer each
            head, head_cuts = A(l, n - 1)
            v = max(head, stage_time(t, mem, budget, n - 1, l + 1, y))
            if v < best:
                best, cuts = v, head_cuts + (y,)
        return best, cuts

    if L < n_dev:
        return INF, None
    return A(L, n_dev)


def layer_partition_bruteforce(t, mem, budget):
    """Every way to cut L layers into len(t) contiguous non-empty stages; returns the least slowest-stage time."""
    n_dev, L = len(t), len(mem)
    best = INF
    for cuts in itertools.combinations(range(1, L), n_dev - 1):
        ends = list(cuts) + [L]
        start, worst = 1, 0.0
        for dev, end in enumerate(ends):
            worst = max(worst, stage_time(t, mem, budget, dev, start, end))
            start = end + 1
        best = min(best, worst)
    return best


# ---- Eq. 2 and 3: tokens into sub-sequences -----------------------------------------------------------
class SequenceDP:
    """W(1..y, k) of Eq. 2 and 3 for one latency function q and one minimum length b, memoised over (y, k).
    granule > 1 restricts the cut points l of Eq. 2 to multiples of granule (every sub-sequence but the last is then a
    whole number of granules); granule = 1 is the recurrence as the paper states it."""

    def __init__(self, q, b, granule=1):
        self.q, self.b, self.granule = q, b, granule
        self._memo = {}

    def t_star(self, x, l):
        return INF if x < self.b else self.q(x, l)

    def W(self, y, k):
        """Returns (W(1..y, k), lengths); ties: the smallest l."""
        key = (y, k)
        if key not in self._memo:
            if k == 1:
                self._memo[key] = (self.t_star(y, 0), (y,))
            else:
                best, lens = INF, None
                for l in range(1, y):
                    if l % self.granule:
                        continue
                    head, head_lens = self.W(l, k - 1)
                    v = max(head, self.t_star(y - l, l))
                    if v < best:
                        best, lens = v, head_lens + (y - l,)
                self._memo[key] = (best, lens)
        return self._memo[key]


def sequence_partition_dp(q, y, k, b, granule=1):
    return SequenceDP(q, b, granule).W(y, k)


def compositions(y, k, b, granule=1):
    """All ways to write y as an ordered sum of k integers >= b, all but the last of them multiples of granule."""
    if k == 1:
        if y >= b:
            yield (y,)
        return
    for first in range(b, y - b * (k - 1) + 1):
        if first % granule:
            continue
        for rest in compositions(y - first, k - 1, b, granule):
            yield (first,) + rest


def chunk_latencies(q, lengths):
    """h_i = q(|s_i|, tokens before s_i)."""
    out, before = [], 0
    for x in lengths:
        out.append(q(x, before))
        before += x
    return out


def sequence_partition_bruteforce(q, y, k, b, granule=1):
    best = INF
    for lens in compositions(y, k, b, granule):
        best = min(best, max(chunk_latencies(q, lens)))
    return best


# ---- Eq. 4: latency of a partition on |D| devices -------------------------------------------------------
def pipeline_latency(q, lengths, n_devices):
    h = chunk_latencies(q, lengths)
    return sum(h) + (n_devices - 1) * max(h)


def choose_k(q, y, b, n_devices, granule=1):
    """k in 1..4|D| minimising Eq. 4 over the partitions of Eq. 2; returns (k, lengths, latency). Ties: smallest k."""
    best = (None, None, INF)
    dp = SequenceDP(q, b, granule)
    for k in range(1, 4 * n_devices + 1):
        w, lens = dp.W(y, k)
        if lens is None or w == INF:
            continue
        lat = pipeline_latency(q, lens, n_devices)
        if lat < best[2]:
            best = (k, lens, lat)
    return best
