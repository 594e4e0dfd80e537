"""Space-filling-curve order of a T x H x W latent grid (test infrastructure only).

This file belongs to the CPU oracle.  Nothing in the product path may import it;
it exists so that tests can check the HIP library against an independent, slow,
readable implementation.

What it follows: Sec. 3.1, Eq. 2 of the paper defines the re-ordering G only as
"an index permutation implemented via generalized Hilbert re-ordering" that
works for cuboids whose sides are not powers of two (appendix, "Index Re-Order
and Block Partition"), and cites a published generalized-Hilbert ("gilbert")
recursion for it.  The paper prints no ordering.  The construction below
restates that published recursion from its description: the same case analysis
(halve a long travel axis, a three-piece planar U when one side axis dominates,
otherwise five pieces along the 8-cell Hilbert path, odd halves raised to even,
line base cases, the planar rule).  What this build adds or chooses itself: the
slab fallback to the planar rule when one length is 1, and the choice of the
outermost travel axis (the longest side, ties w, h, t).  The cited source is not
available here, so equality with its exact ordering is NOT claimed: parity
unpinned.  What carries the curve in the tests are its properties (bijection,
Chebyshev-1 continuity, the 2x2x2 Hilbert cell, the octant property), not
agreement with the host C++ version, which is the same procedure written a
second time.  Everything downstream is defined relative to this order.

Construction.  box(p, A, B, C) visits every cell of the cuboid that has corner p
and signed axis-aligned edge vectors A, B, C (lengths a, b, c >= 1).  It starts
at p and, whenever a > 1, ends at the neighbouring corner along A, p + A - sgn(A).

  * a line (two lengths equal 1) is walked straight;
  * a slab (one length equal 1) is walked by the planar rule in its two
    remaining axes (the longer of them becomes the travel axis when a == 1);
  * if A is long (2a > 3b and 2a > 3c) the box is cut in two across A;
  * if only one of B, C is comparable to A (3b > 4c or 3c > 4b) the box is cut
    into three in the plane of A and the longer side axis: out along that axis
    over the first half of A, across the whole of A, and back;
  * otherwise it is cut into five sub-boxes that follow the 8-cell Hilbert path
    (0,0,0) (0,1,0) (0,1,1) (0,0,1) (1,0,1) (1,1,1) (1,1,0) (1,0,0), with the cell
    pairs that share a face merged.

  Cuts are at floor(n/2), moved up by one when that is odd and n > 2, so that a
  sub-box whose travel axis is the cut length can be crossed corner to adjacent
  corner with unit steps.

The recursion is written with an explicit stack so that the order of emission is
the order of the curve.
"""
import numpy as np


def _sgn(v):
    return (int(v[0] > 0) - int(v[0] < 0),
            int(v[1] > 0) - int(v[1] < 0),
            int(v[2] > 0) - int(v[2] < 0))


def _len(v):
    return abs(v[0]) + abs(v[1]) + abs(v[2])


def _add(*vs):
    return (sum(v[0] for v in vs), sum(v[1] for v in vs), sum(v[2] for v in vs))


def _neg(v):
    return (-v[0], -v[1], -v[2])


def _scale(unit, n):
    return (unit[0] * n, unit[1] * n, unit[2] * n)


def _cut(n):
    h = n // 2
    if h % 2 == 1 and n > 2:
        h += 1
    return h


ZERO = (0, 0, 0)


def _children(p, A, B, C):
    """Return either ('line', p, step, n) or a list of sub-boxes in visiting order."""
    a, b, c = _len(A), _len(B), _len(C)
    dA, dB, dC = _sgn(A), _sgn(B), _sgn(C)

    # lines
    if b == 1 and c == 1:
        return ("line", p, dA, a)
    if a == 1 and c == 1:
        return ("line", p, dB, b)
    if a == 1 and b == 1:
        return ("line", p, dC, c)

    # slabs: fall to the planar rule by giving the flat axis the role of C
    if a == 1:
        if b >= c:
            return [(p, B, C, A)]
        return [(p, C, B, A)]
    if b == 1:
        return _planar(p, A, C, B)
    if c == 1:
        return _planar(p, A, B, C)

    a2, b2, c2 = _cut(a), _cut(b), _cut(c)
    A2, B2, C2 = _scale(dA, a2), _scale(dB, b2), _scale(dC, c2)
    Ar, Br, Cr = _scale(dA, a - a2), _scale(dB, b - b2), _scale(dC, c - c2)
    endA = _add(A, _neg(dA))      # offset of the far corner along A
    endB2 = _add(B2, _neg(dB))
    endC = _add(C, _neg(dC))
    endC2 = _add(C2, _neg(dC))

    if 2 * a > 3 * b and 2 * a > 3 * c:
        return [(p, A2, B, C), (_add(p, A2), Ar, B, C)]
    if 3 * b > 4 * c:
        return [(p, B2, C, A2),
                (_add(p, B2), A, Br, C),
                (_add(p, endA, endB2), _neg(B2), C, _neg(Ar))]
    if 3 * c > 4 * b:
        return [(p, C2, A2, B),
                (_add(p, C2), A, B, Cr),
                (_add(p, endA, endC2), _neg(C2), _neg(Ar), B)]
    return [(p, B2, C2, A2),
            (_add(p, B2), C, A2, Br),
            (_add(p, endB2, endC), A, _neg(B2), _neg(Cr)),
            (_add(p, endA, B2, endC), _neg(C), _neg(Ar), Br),
            (_add(p, endA, endB2), _neg(B2), C2, _neg(Ar))]


def _planar(p, A, B, F):
    """Planar rule for a slab: travel axis A (a > 1), side axis B (b > 1), flat axis F."""
    a, b = _len(A), _len(B)
    dA, dB = _sgn(A), _sgn(B)
    a2, b2 = _cut(a), _cut(b)
    A2, B2 = _scale(dA, a2), _scale(dB, b2)
    Ar, Br = _scale(dA, a - a2), _scale(dB, b - b2)
    if 2 * a > 3 * b:
        return [(p, A2, B, F), (_add(p, A2), Ar, B, F)]
    endA = _add(A, _neg(dA))
    endB2 = _add(B2, _neg(dB))
    return [(p, B2, A2, F),
            (_add(p, B2), A, Br, F),
            (_add(p, endA, endB2), _neg(B2), _neg(Ar), F)]


def curve_cells(T, H, W):
    """Cells (t, h, w) of the T x H x W grid in curve order, as an int array [T*H*W, 3].

    The travel axis of the outermost box is the longest side (ties: w, then h,
    then t), the other two follow in the same preference order.
    """
    if T < 1 or H < 1 or W < 1:
        raise ValueError("grid sides must be >= 1")
    sides = [(W, 2), (H, 1), (T, 0)]            # (length, axis index in (t,h,w))
    order = sorted(range(3), key=lambda i: (-sides[i][0], i))
    vecs = []
    for i in order:
        n, ax = sides[i]
        v = [0, 0, 0]
        v[ax] = n
        vecs.append(tuple(v))
    out = np.empty((T * H * W, 3), dtype=np.int64)
    n_out = 0
    stack = [(ZERO, vecs[0], vecs[1], vecs[2])]
    while stack:
        p, A, B, C = stack.pop()
        kids = _children(p, A, B, C)
        if isinstance(kids, tuple):
            _, q, step, n = kids
            for i in range(n):
                out[n_out, 0] = q[0] + i * step[0]
                out[n_out, 1] = q[1] + i * step[1]
                out[n_out, 2] = q[2] + i * step[2]
                n_out += 1
        else:
            for kid in reversed(kids):
                stack.append(kid)
    assert n_out == T * H * W
    return out


def linear_index(cells, T, H, W):
    """Row-major (t, h, w) index, w fastest: the 'thw' flattening of Sec. 3.1."""
    return (cells[:, 0] * H + cells[:, 1]) * W + cells[:, 2]


def curve_perm(T, H, W, use_curve=True):
    """perm[i] = thw index of the token at curve position i; inv[perm[i]] = i  (Eq. 2).

    use_curve=False gives the identity (the paper's 'linear' partition ablation).
    """
    n = T * H * W
    if not use_curve:
        perm = np.arange(n, dtype=np.int64)
    else:
        perm = linear_index(curve_cells(T, H, W), T, H, W)
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n, dtype=np.int64)
    return perm, inv
