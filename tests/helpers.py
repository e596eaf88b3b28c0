"""Independent re-statements used to pin the oracle (pure Python / numpy, no oracle code).

Nothing here is shared with the HIP path or with ``oracle/``: these are the set-based
definitions of Eq.(7) and exact-rational arithmetic, written out a second time in a
different form so that a mistake in the oracle shows up as a disagreement.
"""
from __future__ import annotations

import bisect
from fractions import Fraction

import numpy as np

NONE, GPU, NODE = 0, 1, 2


# ---------------------------------------------------------------------------
# Eq.(7) by sets: a token goes to a group iff one of its experts lies in the group.
# ---------------------------------------------------------------------------
def brute_plan(ids, w, e2r, nodes, rpn, level):
    """Plan from the set definition.  Rows are the sorted list of (destination, token[, slot])
    tuples -- a global sort instead of the oracle's per-destination cursors.  Slots with the id
    -1 (dropped by the router) take no part in anything."""
    T, K = ids.shape
    G = nodes * rpn
    Dn = nodes if level == NODE else G
    live = [(t, k) for t in range(T) for k in range(K) if ids[t, k] != -1]
    live_k = {t: [k for k in range(K) if ids[t, k] != -1] for t in range(T)}

    def dest(t, k):
        g = int(e2r[ids[t, k]])
        return g // rpn if level == NODE else g

    if level == NONE:
        rows = sorted((dest(t, k), t, k) for t, k in live)
        index = {r: i for i, r in enumerate(rows)}
        slot_row = [[index[(dest(t, k), t, k)] if ids[t, k] != -1 else -1 for k in range(K)] for t in range(T)]
        slot_keep = [[int(ids[t, k] != -1) for k in range(K)] for t in range(T)]
        dest_count = [sum(1 for t, k in live if dest(t, k) == j) for j in range(Dn)]
    else:
        rows = sorted({(dest(t, k), t) for t, k in live})
        index = {r: i for i, r in enumerate(rows)}
        slot_row = [[index[(dest(t, k), t)] if ids[t, k] != -1 else -1 for k in range(K)] for t in range(T)]
        slot_keep = [[int(ids[t, k] != -1 and k == min(k1 for k1 in live_k[t] if dest(t, k1) == dest(t, k)))
                      for k in range(K)] for t in range(T)]
        # duplicate-free count of group j = |{tokens whose group mask is set}|
        dest_count = [len({t for t, k in live if dest(t, k) == j}) for j in range(Dn)]
    row_token = [r[1] for r in rows]
    row_weight = []
    for i, r in enumerate(rows):
        acc = None
        t = r[1]
        for k in range(K):
            if slot_row[t][k] == i:
                acc = np.float32(w[t, k]) if acc is None else np.float32(acc + np.float32(w[t, k]))
        row_weight.append(acc)
    rank_mask = [0] * T
    node_mask = [0] * T
    for t, k in live:
        g = int(e2r[ids[t, k]])
        rank_mask[t] |= 1 << g
        node_mask[t] |= 1 << (g // rpn)
    return dict(dest_count=dest_count, row_token=row_token, slot_row=slot_row, slot_keep=slot_keep,
                row_weight=row_weight, rank_mask=rank_mask, node_mask=node_mask, num_dest=Dn)


def group_counts_by_sets(ids, e2r, n_groups_fn):
    """|{t : some expert of t maps to group j}| for the group map n_groups_fn(rank) -> group."""
    seen = {}
    for t in range(ids.shape[0]):
        for k in range(ids.shape[1]):
            seen.setdefault(n_groups_fn(int(e2r[ids[t, k]])), set()).add(t)
    return {j: len(s) for j, s in seen.items()}


# ---------------------------------------------------------------------------
# bf16 helpers: ordering key for ulp distance, and exact rounding by search
# ---------------------------------------------------------------------------
def bf16_order_key(bits: np.ndarray) -> np.ndarray:
    """Map bf16 encodings to integers that increase with the value (+0 and -0 coincide)."""
    b = bits.astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag)


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    return np.abs(bf16_order_key(a_bits) - bf16_order_key(b_bits))


def _all_finite_bf16():
    enc = np.arange(0x0000, 0x7F80, dtype=np.uint16)            # +0 .. largest finite
    vals = (enc.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return enc, [Fraction(float(v)) for v in vals]


_ENC, _VALS = None, None


def exact_round_to_bf16(q: Fraction) -> int:
    """Nearest bf16 encoding of the rational q, ties to the even encoding, by bisection over the
    table of all finite non-negative bf16 values (no floating-point rounding involved)."""
    global _ENC, _VALS
    if _VALS is None:
        _ENC, _VALS = _all_finite_bf16()
    sign = 0x8000 if q < 0 else 0
    a = -q if q < 0 else q
    i = bisect.bisect_left(_VALS, a)
    if i < len(_VALS) and _VALS[i] == a:
        return sign | int(_ENC[i])
    if i == len(_VALS):                      # above the largest finite value
        top = _VALS[-1]
        half_gap = (top - _VALS[-2]) / 2
        return sign | (0x7F80 if a - top >= half_gap else int(_ENC[-1]))
    lo, hi = _VALS[i - 1], _VALS[i]
    dl, dh = a - lo, hi - a
    if dl < dh:
        pick = i - 1
    elif dh < dl:
        pick = i
    else:
        pick = i - 1 if (int(_ENC[i - 1]) & 1) == 0 else i
    return sign | int(_ENC[pick])


def brute_plan_mapped(ids, w, dest_map, num_dest, dedup):
    """Set-based plan for an arbitrary expert -> destination table (-1 = no copy at this hop)."""
    rows_n, K = ids.shape

    def dest(i, k):
        return int(dest_map[ids[i, k]])

    valid = [(i, k) for i in range(rows_n) for k in range(K) if dest(i, k) >= 0]
    if dedup:
        rows = sorted({(dest(i, k), i) for i, k in valid})
        index = {r: n for n, r in enumerate(rows)}
        slot_row = [[index[(dest(i, k), i)] if dest(i, k) >= 0 else -1 for k in range(K)] for i in range(rows_n)]
        slot_keep = [[int(dest(i, k) >= 0 and k == min(k1 for k1 in range(K) if dest(i, k1) == dest(i, k)))
                      for k in range(K)] for i in range(rows_n)]
        dest_count = [len({i for i, k in valid if dest(i, k) == j}) for j in range(num_dest)]
    else:
        rows = sorted((dest(i, k), i, k) for i, k in valid)
        index = {r: n for n, r in enumerate(rows)}
        slot_row = [[index[(dest(i, k), i, k)] if dest(i, k) >= 0 else -1 for k in range(K)] for i in range(rows_n)]
        slot_keep = [[int(dest(i, k) >= 0) for k in range(K)] for i in range(rows_n)]
        dest_count = [sum(1 for i, k in valid if dest(i, k) == j) for j in range(num_dest)]
    row_weight = []
    for n, r in enumerate(rows):
        acc = None
        for k in range(K):
            if slot_row[r[1]][k] == n:
                acc = np.float32(w[r[1], k]) if acc is None else np.float32(acc + np.float32(w[r[1], k]))
        row_weight.append(acc)
    mask = [0] * rows_n
    for i, k in valid:
        mask[i] |= 1 << dest(i, k)
    return dict(dest_count=dest_count, row_token=[r[1] for r in rows], slot_row=slot_row, slot_keep=slot_keep,
                row_weight=row_weight, dest_mask=mask)


def exact_round_to_f32(q: Fraction) -> float:
    """Nearest binary32 value of the rational q (normal range only), ties to even, in integer
    arithmetic: no floating-point rounding involved."""
    if q == 0:
        return 0.0
    sign = -1 if q < 0 else 1
    a = -q if q < 0 else q
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1) and -126 <= e <= 127
    scaled = a / Fraction(2) ** (e - 23)                  # in [2^23, 2^24)
    n, rem = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * rem
    if twice > scaled.denominator or (twice == scaled.denominator and (n & 1)):
        n += 1
    v = Fraction(n) * Fraction(2) ** (e - 23)
    out = float(v)                                        # exact: at most 24 significant bits
    assert Fraction(out) == v
    return sign * out
