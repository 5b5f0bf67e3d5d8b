"""Generic prefix scans over a monoid -- TEST INFRASTRUCTURE (pure Python, small cases only).

The paper maps attention onto a two-level prefix scan (Sec. 3.2, "Physical
level"): Hillis-Steele inside blocks of B = 128 items, a Blelloch two-pass
(up-sweep / down-sweep) across the block totals.  These routines take any
``(op, identity)`` pair, so the same code is pinned with the integer sum monoid
of the integral-image example (Fig. 1a) and then used with the softmax merge.
Nothing here is shared with, or imported by, the HIP library.
"""
from __future__ import annotations

import math


def sequential_scan(items, op, identity):
    """Inclusive left-to-right scan: out[j] = x_0 (+) ... (+) x_j."""
    out, acc = [], identity
    for x in items:
        acc = op(acc, x)
        out.append(acc)
    return out


def hillis_steele_scan(items, op):
    """Inclusive Hillis-Steele scan: ceil(log2 len) levels, level l combines
    element j with element j - 2^l (all elements active at every level)."""
    cur = list(items)
    n, off = len(cur), 1
    while off < n:
        nxt = list(cur)
        for j in range(off, n):
            nxt[j] = op(cur[j - off], cur[j])
        cur, off = nxt, off * 2
    return cur


def blelloch_exclusive_scan(items, op, identity):
    """Blelloch work-efficient exclusive scan (up-sweep then down-sweep), padded
    with the identity to a power of two.  Returns (exclusive prefixes, total)."""
    n = len(items)
    if n == 0:
        return [], identity
    size = 1 << max(0, (n - 1).bit_length())
    a = list(items) + [identity] * (size - n)
    step = 1
    while step < size:                       # up-sweep: build partial totals
        for j in range(2 * step - 1, size, 2 * step):
            a[j] = op(a[j - step], a[j])
        step *= 2
    total = a[size - 1]
    a[size - 1] = identity                   # the identity seeds the down-sweep
    step = size // 2
    while step >= 1:                         # down-sweep: distribute prefixes
        for j in range(2 * step - 1, size, 2 * step):
            left = a[j - step]
            a[j - step] = a[j]
            a[j] = op(a[j], left)            # prefix (+) left subtree, order preserved
        step //= 2
    return a[:n], total


def two_level_scan(items, op, identity, block=128):
    """The paper's two-level scan: inclusive Hillis-Steele within each block,
    Blelloch exclusive scan over block totals, block prefix (+) local state."""
    blocks = [list(items[s:s + block]) for s in range(0, len(items), block)]
    local = [hillis_steele_scan(b, op) for b in blocks]
    totals = [l[-1] for l in local]
    prefixes, total = blelloch_exclusive_scan(totals, op, identity)
    out = []
    for pre, loc in zip(prefixes, local):
        out.extend(op(pre, x) for x in loc)
    return out, total


def merge_depth(n, block=128):
    """L(n, B) = ceil(log2 B) + 2 ceil(log2(n / B)) + 3   (Eq. 5)."""
    inter = max(0, math.ceil(math.log2(max(1.0, n / block))))
    return math.ceil(math.log2(block)) + 2 * inter + 3
