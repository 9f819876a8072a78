"""GPU parity: dc_match_blocks against the oracle, bit-exact (Section 4, Steps 1-4)."""
import numpy as np
import pytest
import torch

from paper_1712_01670_amd import binding, synth

pytestmark = pytest.mark.gpu


def _run(cur, prev, B, R, thr):
    """cur, prev: numpy uint8 [n][H][W][C]"""
    dev = torch.device("cuda:0")
    out = binding.dc_match_blocks(torch.from_numpy(cur).to(dev), torch.from_numpy(prev).to(dev), B, R, thr)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def _compare(oracle, cur, prev, B, R, thr, tag):
    print(f"[match] {tag} shape={cur.shape} B={B} R={R} thr={thr}", flush=True)
    got = _run(cur, prev, B, R, thr)
    for s in range(cur.shape[0]):
        want = oracle.match_blocks(cur[s], prev[s], B, R, thr)
        assert np.array_equal(got["best_ssd"][s].view(np.uint32), want["best_ssd"]), (tag, s)
        assert np.array_equal(got["mv"][s], want["mv"]), (tag, s)
        assert got["gmv"][s].tolist() == want["gmv"].tolist(), (tag, s)
        assert int(got["n_pass"][s]) == want["n_pass"], (tag, s)
        assert np.array_equal(got["mask"][s], want["mask"]), (tag, s)


def test_tiny_config(oracle):
    f1, f2 = synth.tiny_pair(0)
    _compare(oracle, f2[None], f1[None], 8, 8, synth.max_block_ssd(8), "tiny")


def test_identical_and_unrelated_frames(oracle):
    rng = np.random.default_rng(0)
    a = rng.integers(0, 256, (2, 64, 96, 3)).astype(np.uint8)
    b = rng.integers(0, 256, (2, 64, 96, 3)).astype(np.uint8)
    _compare(oracle, a, a, 16, 16, 0, "identical")
    _compare(oracle, a, b, 16, 16, 100, "unrelated")
    flat = np.full((1, 64, 64, 3), 9, np.uint8)
    _compare(oracle, flat, flat, 8, 8, 0, "flat ties")


def test_tie_break_patterns(oracle):
    prev = np.zeros((1, 32, 32, 3), np.uint8)
    prev[0, 1::2] = 200
    cur = np.zeros((1, 32, 32, 3), np.uint8)
    cur[0, 0::2] = 200
    _compare(oracle, cur, prev, 8, 4, 0, "h stripes")
    _compare(oracle, np.ascontiguousarray(cur.transpose(0, 2, 1, 3)),
             np.ascontiguousarray(prev.transpose(0, 2, 1, 3)), 8, 4, 0, "v stripes")
    yy, xx = np.mgrid[0:32, 0:32]
    p = np.repeat((((yy + xx) % 2) * 200).astype(np.uint8)[None, :, :, None], 3, 3)
    _compare(oracle, 200 - p, p, 8, 4, 0, "checker")


def test_panning_video_vgg_geometry(oracle):
    fr = synth.panning_video(2000, n_frames=4)
    _compare(oracle, fr[1:4], fr[0:3], 16, 16, synth.max_block_ssd(16), "panning 224 (3 streams)")


@pytest.mark.parametrize("H,W,C,B,R", [(50, 70, 3, 10, 7), (45, 53, 1, 5, 3), (40, 44, 4, 8, 8),
                                       (227, 227, 3, 10, 8), (33, 35, 3, 16, 16), (64, 64, 2, 7, 5)])
def test_ragged_shapes_and_unaligned_rows(oracle, H, W, C, B, R):
    rng = np.random.default_rng(H * W)
    prev = synth._box_blur5(rng.integers(0, 256, (H, W, C)).astype(np.uint8))
    cur = np.roll(prev, (2, -3), axis=(0, 1))
    cur[H // 2:H // 2 + B, W // 3:W // 3 + B] = rng.integers(0, 256, (min(B, H - H // 2), min(B, W - W // 3), C))
    _compare(oracle, cur[None], prev[None], B, R, 30 * B * B * C, f"ragged {H}x{W}x{C}")


def test_extreme_values_do_not_overflow(oracle):
    a = np.zeros((1, 64, 64, 3), np.uint8)
    b = np.full((1, 64, 64, 3), 255, np.uint8)
    _compare(oracle, a, b, 16, 16, 2 ** 32 - 1, "0 vs 255")
    _compare(oracle, b, a, 16, 16, 0, "255 vs 0")


def test_darknet_geometry_sampled(oracle):
    # full-size 416x416 frame pair; the oracle checks everything (676 blocks, a few seconds)
    fr = synth.reuse_sweep_video(4002, 0.5, n_frames=2)
    _compare(oracle, fr[1:2], fr[0:1], 16, 16, synth.max_block_ssd(16), "sweep 416")


@pytest.mark.parametrize("k", [2, 3])
def test_k_skip(oracle, k):
    """Exhaustive search on every k-th block row and column only (the acceleration at the end of Section 4)."""
    dev = torch.device("cuda:0")
    fr = synth.panning_video(2000, n_frames=4)
    cases = [(fr[1:4], fr[0:3], 16, 16, synth.max_block_ssd(16))]
    rng = np.random.default_rng(k)
    prev = synth._box_blur5(rng.integers(0, 256, (1, 50, 70, 3)).astype(np.uint8).reshape(50, 70, 3))[None]
    cur = np.roll(prev, (2, -3), axis=(1, 2))
    cases.append((cur, prev, 10, 7, 30 * 300))
    cases.append((cur, prev, 10, 7, 2 ** 32 - 1))          # the bound does not make skipped blocks count
    for cur, prev, B, R, thr in cases:
        print(f"[match k-skip] k={k} shape={cur.shape} B={B} R={R} thr={thr}", flush=True)
        out = binding.dc_match_blocks_opt(torch.from_numpy(np.ascontiguousarray(cur)).to(dev),
                                          torch.from_numpy(np.ascontiguousarray(prev)).to(dev), B, R, thr,
                                          method=binding.DC_MATCH_EXHAUSTIVE, k_skip=k)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
        for s in range(cur.shape[0]):
            want = oracle.match_blocks(cur[s], prev[s], B, R, thr, k_skip=k)
            assert np.array_equal(got["best_ssd"][s].view(np.uint32), want["best_ssd"])
            assert np.array_equal(got["mv"][s], want["mv"])
            assert got["gmv"][s].tolist() == want["gmv"].tolist()
            assert int(got["n_pass"][s]) == want["n_pass"]
            assert np.array_equal(got["mask"][s], want["mask"])
