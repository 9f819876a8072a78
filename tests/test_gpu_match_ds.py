"""GPU parity: dc_match_blocks_ds (diamond search, k-skip) against the oracle, bit-exact
(Section 4, Steps 1-4 with the search the paper runs in Step 2)."""
import numpy as np
import pytest
import torch

from paper_1712_01670_amd import binding, synth

pytestmark = pytest.mark.gpu


def _run(cur, prev, B, R, thr, k):
    dev = torch.device("cuda:0")
    out = binding.dc_match_blocks_ds(torch.from_numpy(cur).to(dev), torch.from_numpy(prev).to(dev), B, R, thr, k)
    torch.cuda.synchronize()
    return {key: v.cpu().numpy() for key, v in out.items()}


def _compare(oracle, cur, prev, B, R, thr, tag, ks=(1, 2, 3)):
    for k in ks:
        print(f"[match ds] {tag} shape={cur.shape} B={B} R={R} thr={thr} k={k}", flush=True)
        got = _run(cur, prev, B, R, thr, k)
        for s in range(cur.shape[0]):
            want = oracle.match_blocks_ds(cur[s], prev[s], B, R, thr, k_skip=k)
            assert np.array_equal(got["best_ssd"][s].view(np.uint32), want["best_ssd"]), (tag, k, s)
            assert np.array_equal(got["mv"][s], want["mv"]), (tag, k, s)
            assert got["gmv"][s].tolist() == want["gmv"].tolist(), (tag, k, s)
            assert int(got["n_pass"][s]) == want["n_pass"], (tag, k, s)
            assert np.array_equal(got["mask"][s], want["mask"]), (tag, k, s)


def test_tiny_config(oracle):
    f1, f2 = synth.tiny_pair(0)
    _compare(oracle, f2[None], f1[None], 8, 8, synth.max_block_ssd(8), "tiny")


def test_identical_unrelated_and_flat_frames(oracle):
    rng = np.random.default_rng(0)
    a = rng.integers(0, 256, (2, 64, 96, 3)).astype(np.uint8)
    b = rng.integers(0, 256, (2, 64, 96, 3)).astype(np.uint8)
    _compare(oracle, a, a, 16, 16, 0, "identical")
    _compare(oracle, a, b, 16, 16, 100, "unrelated")
    _compare(oracle, a, b, 16, 16, 2 ** 32 - 1, "unrelated, every searched block passes")
    flat = np.full((1, 64, 64, 3), 9, np.uint8)
    _compare(oracle, flat, flat, 8, 8, 0, "flat: every point ties, the centre stays")


def test_tie_patterns(oracle):
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
    fr = synth.panning_video(2000, n_frames=6)
    _compare(oracle, fr[1:6], fr[0:5], 16, 16, synth.max_block_ssd(16), "panning 224 (5 streams)")
    # the walk follows the pan: most blocks end on the background's vector
    got = _run(fr[1:2], fr[0:1], 16, 16, synth.max_block_ssd(16), 1)
    assert int(got["n_pass"][0]) > 0.5 * 14 * 14


@pytest.mark.parametrize("H,W,C,B,R", [(50, 70, 3, 10, 7), (45, 53, 1, 5, 3), (40, 44, 4, 8, 8),
                                       (227, 227, 3, 10, 8), (33, 35, 3, 16, 16), (64, 64, 2, 7, 5),
                                       (96, 128, 3, 32, 40), (64, 64, 3, 8, 0), (64, 64, 3, 8, 1),
                                       (120, 136, 3, 16, 70), (20, 24, 1, 1, 3)])   # the last one: window too large for LDS
def test_ragged_shapes_long_walks_and_small_ranges(oracle, H, W, C, B, R):
    rng = np.random.default_rng(H * W + R)
    prev = synth._box_blur5(synth._box_blur5(rng.integers(0, 256, (H, W, C)).astype(np.uint8)))
    cur = np.roll(prev, (5, -6), axis=(0, 1))      # several rounds of the large pattern
    cur[H // 2:H // 2 + B, W // 3:W // 3 + B] = rng.integers(0, 256, (min(B, H - H // 2), min(B, W - W // 3), C))
    _compare(oracle, cur[None], prev[None], B, R, 30 * B * B * C, f"ragged {H}x{W}x{C}")


def test_extreme_values_do_not_overflow(oracle):
    a = np.zeros((1, 64, 64, 3), np.uint8)
    b = np.full((1, 64, 64, 3), 255, np.uint8)
    _compare(oracle, a, b, 16, 16, 2 ** 32 - 1, "0 vs 255")
    _compare(oracle, b, a, 16, 16, 0, "255 vs 0")


def test_darknet_geometry_many_streams(oracle):
    rng = np.random.default_rng(77)
    base = synth._box_blur5(rng.integers(0, 256, (420, 420, 3)).astype(np.uint8))
    cur = np.stack([np.ascontiguousarray(base[2:418, 2:418]) for _ in range(3)])
    prev = np.stack([np.ascontiguousarray(base[2 + dy:418 + dy, 2 + dx:418 + dx]) for dx, dy in [(2, 0), (-1, 2), (0, 0)]])
    _compare(oracle, cur, prev, 16, 16, synth.max_block_ssd(16), "416x416, 3 streams", ks=(1, 2))


def test_argument_checks():
    dev = torch.device("cuda:0")
    f = torch.zeros((1, 32, 32, 3), dtype=torch.uint8, device=dev)
    with pytest.raises(binding.DcError) as e:
        binding.dc_match_blocks_ds(f, f, 8, 8, 0, k_skip=0)
    assert e.value.status == -1
