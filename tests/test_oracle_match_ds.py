"""Pins for the oracle's diamond-search matcher (Section 4, Step 2 as the paper runs it, with the
k-skip acceleration): walks worked out by hand on small cost tables, invariants that hold for the
published algorithm on any input (checked against an independent numpy cost table), agreement with
the exhaustive search where the cost surface has one basin, and the k-skip bookkeeping."""
from fractions import Fraction

import numpy as np

INVALID = 0xFFFFFFFF
LARGE = [(0, -2), (-1, -1), (1, -1), (-2, 0), (2, 0), (-1, 1), (1, 1), (0, 2)]
SMALL = [(0, -1), (-1, 0), (1, 0), (0, 1)]


def _table(R, fn):
    t = np.zeros((2 * R + 1, 2 * R + 1), np.uint32)
    for dy in range(-R, R + 1):
        for dx in range(-R, R + 1):
            t[dy + R, dx + R] = fn(dx, dy)
    return t


def test_walks_worked_by_hand(oracle):
    # A. bowl at the origin: the first large pattern already has its best point at the centre
    assert oracle.diamond_search_table(_table(4, lambda dx, dy: 10 * (dx * dx + dy * dy))) == ((0, 0), 0, 1)
    # B. bowl at (3,1), cost (dx-3)^2 + (dy-1)^2.  Round 1 around (0,0) [cost 10]: (2,0) -> 2 is the smallest
    #    ((1,1) -> 4, (1,-1) -> 8, (0,2) -> 10, ...).  Round 2 around (2,0): (3,1) -> 0.  Round 3: centre stays.
    assert oracle.diamond_search_table(_table(4, lambda dx, dy: (dx - 3) ** 2 + (dy - 1) ** 2)) == ((3, 1), 0, 3)
    # C. bowl at (1,0): in round 1 the centre costs 1 and (2,0), (1,-1), (1,1) also cost 1: equal cost does not
    #    move the centre; the small pattern then reaches (1,0) -> 0
    assert oracle.diamond_search_table(_table(4, lambda dx, dy: (dx - 1) ** 2 + dy * dy)) == ((1, 0), 0, 1)
    # D. a far, isolated global minimum is not found (this is what separates the method from exhaustive search)
    t = _table(4, lambda dx, dy: 5 + dx * dx + dy * dy)
    t[4 + 4, 4 + 4] = 0
    assert oracle.diamond_search_table(t) == ((0, 0), 5, 1)
    # E. two equal best points of the large pattern: the earlier one in raster order (dy, then dx) wins
    t = _table(4, lambda dx, dy: 100)
    t[-1 + 4, -1 + 4] = 50
    t[1 + 4, 1 + 4] = 50
    assert oracle.diamond_search_table(t) == ((-1, -1), 50, 2)
    # F. the bowl's centre (4,0) lies outside the search range R = 2: the walk stops at the range limit.
    #    Round 1: (2,0) -> 4.  Round 2 around (2,0): (4,0), (3,+-1) are out of range, (2,+-2) -> 8: stays.
    #    Small pattern: (3,0) out of range, (2,+-1) -> 5, (1,0) -> 9: stays.
    assert oracle.diamond_search_table(_table(2, lambda dx, dy: (dx - 4) ** 2 + dy * dy)) == ((2, 0), 4, 2)
    # G. vectors whose window leaves the frame (here every dx < 0) are never taken
    t = _table(2, lambda dx, dy: INVALID if dx < 0 else (dx + 2) ** 2 + dy * dy)
    assert oracle.diamond_search_table(t) == ((0, 0), 4, 1)


def _np_ssd_table(cur, prev, B, R, bx, by):
    H, W, _ = cur.shape
    x, y = bx * B, by * B
    a = cur[y:y + B, x:x + B].astype(np.int64)
    out = {}
    for dy in range(-R, R + 1):
        for dx in range(-R, R + 1):
            if x + dx < 0 or y + dy < 0 or x + dx + B > W or y + dy + B > H:
                continue
            b = prev[y + dy:y + dy + B, x + dx:x + dx + B].astype(np.int64)
            out[(dx, dy)] = int(((a - b) ** 2).sum())
    return out


def _is_diamond_fixed_point(tab, mv):
    """mv is the best small-pattern point of some centre that is itself the best of its large pattern."""
    for c in [mv] + [(mv[0] - dx, mv[1] - dy) for dx, dy in SMALL]:
        if c not in tab:
            continue
        large = [tab[(c[0] + dx, c[1] + dy)] for dx, dy in LARGE if (c[0] + dx, c[1] + dy) in tab]
        small = [tab[(c[0] + dx, c[1] + dy)] for dx, dy in SMALL if (c[0] + dx, c[1] + dy) in tab]
        if all(tab[c] <= v for v in large) and tab[mv] == min([tab[c]] + small):
            return True
    return False


def test_invariants_on_random_frames(oracle):
    rng = np.random.default_rng(11)
    for B, R, (H, W), C in [(4, 3, (16, 20), 3), (8, 6, (40, 48), 3), (5, 4, (23, 27), 1)]:
        prev = rng.integers(0, 256, (H, W, C)).astype(np.uint8)
        cur = rng.integers(0, 256, (H, W, C)).astype(np.uint8)
        ds = oracle.match_blocks_ds(cur, prev, B, R, 10 ** 9)
        es = oracle.match_blocks(cur, prev, B, R, 10 ** 9)
        for by in range(H // B):
            for bx in range(W // B):
                tab = _np_ssd_table(cur, prev, B, R, bx, by)
                mv = tuple(int(v) for v in ds["mv"][by, bx])
                assert mv in tab and ds["best_ssd"][by, bx] == tab[mv]
                assert tab[mv] <= tab[(0, 0)]                       # never worse than no motion
                assert tab[mv] >= es["best_ssd"][by, bx]            # never better than the exhaustive search
                assert _is_diamond_fixed_point(tab, mv)
                assert ds["rounds"][by, bx] >= 1


def _moved(seed, H, W, shift, C=3):
    """Blurred noise and the same content moved by `shift` = (right, down), cut from one larger canvas."""
    from paper_1712_01670_amd import synth
    pad = 8
    big, _ = synth.shifted_pair(seed, H + 2 * pad, W + 2 * pad, (0, 0), C)
    f1 = big[pad:pad + H, pad:pad + W]
    f2 = big[pad - shift[1]:pad - shift[1] + H, pad - shift[0]:pad - shift[0] + W]
    return np.ascontiguousarray(f1), np.ascontiguousarray(f2)


def test_motion_on_the_large_pattern_is_found_in_two_rounds(oracle):
    # content moved by a point of the large pattern: round 1 sees cost 0 there and every other point costs
    # more, round 2 keeps the centre, the small pattern keeps it too.  The exhaustive search finds the same.
    for i, (dx, dy) in enumerate(LARGE):
        f1, f2 = _moved(20 + i, 48, 64, (-dx, -dy))          # the match of a block lies at (dx, dy)
        ds = oracle.match_blocks_ds(f2, f1, 8, 8, 0)
        es = oracle.match_blocks(f2, f1, 8, 8, 0)
        gy, gx = np.mgrid[0:6, 0:8]
        inside = (gx * 8 + dx >= 0) & (gx * 8 + dx + 8 <= 64) & (gy * 8 + dy >= 0) & (gy * 8 + dy + 8 <= 48)
        assert (ds["mv"][inside] == np.array([dx, dy])).all()
        assert not ds["best_ssd"][inside].any() and (ds["rounds"][inside] == 2).all()
        assert ds["best_ssd"][~inside].all()                   # the blocks at the edge the content came from
        assert np.array_equal(ds["mv"][inside], es["mv"][inside]) and np.array_equal(ds["mask"], es["mask"])
        assert ds["gmv"].tolist() == [dx, dy] and ds["n_pass"] == int(inside.sum())
        assert np.array_equal(ds["mask"].astype(bool), inside)
    # moved by a point of the small pattern, seen from a frame edge where the walk cannot leave the frame:
    # the top-left block of content moved by (+1, 0) has its match at (-1, 0), outside the frame
    f1, f2 = _moved(40, 48, 64, (1, 0))
    ds = oracle.match_blocks_ds(f2, f1, 8, 8, 10 ** 9)
    tab = _np_ssd_table(f2, f1, 8, 8, 0, 0)
    assert (-1, 0) not in tab and tuple(ds["mv"][0, 0]) in tab and ds["mv"][0, 0][0] >= 0


def test_identical_frames(oracle):
    rng = np.random.default_rng(3)
    f = rng.integers(0, 256, (48, 64, 3)).astype(np.uint8)
    m = oracle.match_blocks_ds(f, f, 8, 8, 0)
    assert not m["mv"].any() and not m["best_ssd"].any() and (m["rounds"] == 1).all()
    assert m["gmv"].tolist() == [0, 0] and m["n_pass"] == 48 and m["mask"].all()


def _round_half_away(fr):
    n, d = fr.numerator, fr.denominator
    q = (2 * abs(n) + d) // (2 * d)
    return -q if n < 0 else q


def test_k_skip(oracle):
    rng = np.random.default_rng(5)
    f1, f2 = _moved(6, 72, 88, (1, -1))
    f2 = f2.copy()
    f2[16:32, 40:56] = rng.integers(0, 256, (16, 16, 3))          # a changed patch
    full = oracle.match_blocks_ds(f2, f1, 8, 8, 300)
    for k in (2, 3):
        m = oracle.match_blocks_ds(f2, f1, 8, 8, 300, k_skip=k)
        gh, gw = 9, 11
        searched = np.zeros((gh, gw), bool)
        searched[::k, ::k] = True
        assert np.array_equal(m["mv"][searched], full["mv"][searched])
        assert np.array_equal(m["best_ssd"][searched], full["best_ssd"][searched])
        assert not m["mv"][~searched].any() and (m["best_ssd"][~searched] == INVALID).all()
        assert not m["rounds"][~searched].any() and (m["rounds"][searched] >= 1).all()
        ok = searched & (m["best_ssd"] <= 300)
        assert m["n_pass"] == int(ok.sum()) > 0
        mx = _round_half_away(Fraction(int(m["mv"][..., 0][ok].sum()), int(ok.sum())))
        my = _round_half_away(Fraction(int(m["mv"][..., 1][ok].sum()), int(ok.sum())))
        assert m["gmv"].tolist() == [mx, my]
        # Step 4 looks at every block, searched or not
        for by in range(gh):
            for bx in range(gw):
                tab = _np_ssd_table(f2, f1, 8, 8, bx, by)
                assert m["mask"][by, bx] == int((mx, my) in tab and tab[(mx, my)] <= 300)
        assert m["mask"][~searched].any()
    # a bound of 2^32-1 does not make the skipped blocks count
    m = oracle.match_blocks_ds(f2, f1, 8, 8, INVALID, k_skip=2)
    assert m["n_pass"] == 5 * 6


def test_k_skip_with_exhaustive_search(oracle):
    # the same bookkeeping with the exhaustive search in Step 2 (the acceleration does not depend on the search)
    rng = np.random.default_rng(9)
    f1, f2 = _moved(8, 72, 88, (-2, 3))
    f2 = f2.copy()
    f2[40:56, 16:40] = rng.integers(0, 256, (16, 24, 3))
    full = oracle.match_blocks(f2, f1, 8, 6, 300)
    assert np.array_equal(oracle.match_blocks(f2, f1, 8, 6, 300, k_skip=1)["mv"], full["mv"])
    for k in (2, 4):
        m = oracle.match_blocks(f2, f1, 8, 6, 300, k_skip=k)
        searched = np.zeros((9, 11), bool)
        searched[::k, ::k] = True
        assert np.array_equal(m["mv"][searched], full["mv"][searched])
        assert np.array_equal(m["best_ssd"][searched], full["best_ssd"][searched])
        assert not m["mv"][~searched].any() and (m["best_ssd"][~searched] == INVALID).all()
        ok = searched & (m["best_ssd"] <= 300)
        assert m["n_pass"] == int(ok.sum()) > 0
        mx = _round_half_away(Fraction(int(m["mv"][..., 0][ok].sum()), int(ok.sum())))
        my = _round_half_away(Fraction(int(m["mv"][..., 1][ok].sum()), int(ok.sum())))
        assert m["gmv"].tolist() == [mx, my] == [2, -3]
        for by in range(9):
            for bx in range(11):
                tab = _np_ssd_table(f2, f1, 8, 6, bx, by)
                assert m["mask"][by, bx] == int((mx, my) in tab and tab[(mx, my)] <= 300)
