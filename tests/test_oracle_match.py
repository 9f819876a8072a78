"""Pins for the oracle's matcher (Section 4, Steps 1-4): closed forms on constructed
frame pairs, the arg-min definition by an independent numpy brute force, the
tie-break and rounding readings by hand cases."""
from fractions import Fraction

import numpy as np

from paper_1712_01670_amd import synth


def _np_ssd_table(cur, prev, B, R, bx, by):
    """Independent brute force: SSD of one block against every in-frame candidate."""
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


def test_identical_frames_give_full_reuse(oracle):
    rng = np.random.default_rng(0)
    f = rng.integers(0, 256, (48, 64, 3)).astype(np.uint8)
    m = oracle.match_blocks(f, f, 8, 8, 0)
    assert not m["mv"].any() and not m["best_ssd"].any()
    assert m["gmv"].tolist() == [0, 0] and m["n_pass"] == 6 * 8
    assert m["mask"].all()


def test_argmin_definition_random(oracle):
    rng = np.random.default_rng(1)
    for B, R, (H, W) in [(4, 3, (16, 20)), (8, 5, (24, 32)), (5, 4, (23, 27))]:
        prev = rng.integers(0, 256, (H, W, 3)).astype(np.uint8)
        cur = rng.integers(0, 256, (H, W, 3)).astype(np.uint8)
        m = oracle.match_blocks(cur, prev, B, R, 10 ** 9)
        assert m["mv"].shape == (H // B, W // B, 2)
        for by in range(H // B):
            for bx in range(W // B):
                tab = _np_ssd_table(cur, prev, B, R, bx, by)
                best = min(tab.items(), key=lambda kv: (kv[1], abs(kv[0][0]) + abs(kv[0][1]), kv[0][1], kv[0][0]))
                assert tuple(m["mv"][by, bx]) == best[0]
                assert m["best_ssd"][by, bx] == best[1]


def test_exact_translation_closed_form(oracle):
    # content moves by (+5 right, -3 up): a block's match in the previous frame is at (-5,+3)
    f1, f2 = synth.shifted_pair(3, 64, 80, (5, -3))
    m = oracle.match_blocks(f2, f1, 8, 8, 0)
    gh, gw = 8, 10
    inner = m["mv"][1:gh - 1, 1:gw - 1].reshape(-1, 2)
    assert (inner == np.array([-5, 3])).all()
    assert not m["best_ssd"][1:gh - 1, 1:gw - 1].any()
    assert m["gmv"].tolist() == [-5, 3]
    # Step 4: exactly the blocks whose source window is in-frame are reusable:
    # left column needs x-5 >= 0 (fails), bottom row needs y+3+8 <= 64 (fails)
    want = np.ones((gh, gw), np.uint8)
    want[:, 0] = 0
    want[gh - 1, :] = 0
    assert np.array_equal(m["mask"], want)


def test_tiny_config_closed_form(oracle):
    # 64x64 pair: shift (+3,-2), sigma-2 noise, fresh 16x16 patch at (24,24); B=8, R=8, tau=20
    f1, f2 = synth.tiny_pair(0)
    m = oracle.match_blocks(f2, f1, 8, 8, synth.max_block_ssd(8))
    assert m["gmv"].tolist() == [-3, 2]
    want = np.ones((8, 8), np.uint8)
    want[:, 0] = 0          # source x-3 < 0
    want[7, :] = 0          # source y+2+8 > 64
    want[3:5, 3:5] = 0      # fresh-noise patch
    assert np.array_equal(m["mask"], want)
    assert int(m["mask"].sum()) == 45
    # interior blocks away from the patch found the true vector
    for by in range(1, 7):
        for bx in range(1, 8):
            if 3 <= by <= 4 and 3 <= bx <= 4:
                continue
            assert tuple(m["mv"][by, bx]) == (-3, 2)


def test_tie_break_prefers_small_then_dy_then_dx(oracle):
    # flat frames: every candidate has SSD 0 -> (0,0)
    f = np.full((32, 32, 3), 77, np.uint8)
    m = oracle.match_blocks(f, f, 8, 4, 0)
    assert not m["mv"].any()
    # horizontal stripes of period 2, current = previous moved by one row:
    # SSD 0 exactly for odd dy (any dx); smallest |dx|+|dy| is dy=+-1, dx=0; tie -> dy=-1
    prev = np.zeros((32, 32, 3), np.uint8)
    prev[1::2] = 200
    cur = np.zeros((32, 32, 3), np.uint8)
    cur[0::2] = 200
    m = oracle.match_blocks(cur, prev, 8, 4, 0)
    assert (m["mv"][1:, :, 0] == 0).all() and (m["mv"][1:, :, 1] == -1).all()
    assert (m["mv"][0, :, 1] == 1).all()      # top row: dy=-1 is out of frame
    # vertical stripes: SSD 0 for odd dx; dy=0; tie between dx=-1 and dx=+1 -> dx=-1
    m = oracle.match_blocks(np.ascontiguousarray(cur.transpose(1, 0, 2)),
                            np.ascontiguousarray(prev.transpose(1, 0, 2)), 8, 4, 0)
    assert (m["mv"][:, 1:, 0] == -1).all() and (m["mv"][:, 1:, 1] == 0).all()
    assert (m["mv"][:, 0, 0] == 1).all()
    # checkerboard of period 2: SSD 0 iff dx+dy odd: candidates (0,-1),(−1,0),(1,0),(0,1)
    # all have |dx|+|dy| = 1; smallest dy wins -> (0,-1)
    yy, xx = np.mgrid[0:32, 0:32]
    prev = np.repeat((((yy + xx) % 2) * 200).astype(np.uint8)[:, :, None], 3, 2)
    cur = 200 - prev
    m = oracle.match_blocks(cur, prev, 8, 4, 0)
    assert (m["mv"][1:, :, 0] == 0).all() and (m["mv"][1:, :, 1] == -1).all()
    assert (m["mv"][0, 1:, 0] == -1).all() and (m["mv"][0, 1:, 1] == 0).all()
    assert tuple(m["mv"][0, 0]) == (1, 0)


def _round_half_away(fr):
    s = -1 if fr < 0 else 1
    fr = abs(fr)
    n = fr.numerator // fr.denominator
    rem = fr - n
    return s * (n + (1 if rem >= Fraction(1, 2) else 0))


def test_global_motion_is_rounded_mean_over_passing_blocks(oracle):
    rng = np.random.default_rng(5)
    base = synth._box_blur5(rng.integers(0, 256, (64, 96, 3)).astype(np.uint8))
    # left half moves by 1 px left, right half stays: mean motion is fractional
    for split, shift in [(48, 1), (48, -1), (32, 1), (64, -2), (16, 1)]:
        cur = base.copy()
        cur[:, :split] = np.roll(base, -shift, axis=1)[:, :split]
        m = oracle.match_blocks(cur, base, 8, 4, 30 * 8 * 8 * 3)
        ok = m["best_ssd"] <= 30 * 8 * 8 * 3
        K = int(ok.sum())
        assert K == m["n_pass"] and K > 0
        sx = int(m["mv"][..., 0][ok].astype(np.int64).sum())
        sy = int(m["mv"][..., 1][ok].astype(np.int64).sum())
        assert m["gmv"].tolist() == [_round_half_away(Fraction(sx, K)), _round_half_away(Fraction(sy, K))]
    # exact halves: 2 blocks, one moved by +1 -> mean +0.5 -> +1 ; by -1 -> -0.5 -> -1
    for shift, want in [(1, 1), (-1, -1)]:
        prev = synth._box_blur5(rng.integers(0, 256, (8, 40, 3)).astype(np.uint8))
        cur = prev.copy()
        # block 1 of 5 (x in 8..16) shows content from x+shift; others unchanged;
        # restrict to two passing blocks by ruining blocks 2..4
        cur[:, 8:16] = prev[:, 8 + shift:16 + shift]
        cur[:, 16:] = 255 - cur[:, 16:]
        m = oracle.match_blocks(cur, prev, 8, 3, 0)
        assert m["n_pass"] == 2 and m["gmv"].tolist() == [want, 0]


def test_no_passing_block_means_no_reuse(oracle):
    rng = np.random.default_rng(9)
    a = rng.integers(0, 256, (32, 32, 3)).astype(np.uint8)
    b = rng.integers(0, 256, (32, 32, 3)).astype(np.uint8)
    m = oracle.match_blocks(a, b, 8, 4, 100)
    assert m["n_pass"] == 0 and not m["mask"].any() and m["gmv"].tolist() == [0, 0]


def test_retest_uses_global_vector_not_best_vector(oracle):
    # Step 4: a block whose own best vector differs from the global motion is reusable
    # only if it also matches at the global motion (moving object -> not reusable)
    rng = np.random.default_rng(11)
    prev = synth._box_blur5(rng.integers(0, 256, (64, 64, 3)).astype(np.uint8))
    cur = prev.copy()
    obj = rng.integers(0, 256, (8, 8, 3)).astype(np.uint8)
    prev[16:24, 16:24] = obj          # object sits here in the previous frame
    cur[16:24, 24:32] = obj           # and one block to the right in the current frame
    m = oracle.match_blocks(cur, prev, 8, 8, 0)
    assert m["gmv"].tolist() == [0, 0]
    assert tuple(m["mv"][2, 3]) == (-8, 0) and m["best_ssd"][2, 3] == 0
    assert m["mask"][2, 3] == 0       # best match passes, re-test at (0,0) fails
    assert m["mask"][2, 2] == 0       # uncovered background
    assert m["mask"].sum() == 62


def test_remainder_strip_is_ignored(oracle):
    rng = np.random.default_rng(13)
    f = rng.integers(0, 256, (27, 29, 3)).astype(np.uint8)
    m = oracle.match_blocks(f, f, 10, 4, 0)
    assert m["mask"].shape == (2, 2) and m["mask"].all()
