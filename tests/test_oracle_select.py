"""Pins for the oracle's A2 selection (Sec. III-B, selective fine inference).

Each test checks the oracle against something other than itself: the two
limiting cases the definition fixes (no RoI -> coarse grid, RoI everywhere ->
fine grid), exact tiling of the frame, a per-pixel brute force that never
intersects rectangles, and hand-worked examples.
"""
import numpy as np
import pytest

from oracle import cfdetr_oracle as O
from paper_2505_23317_amd import synth


def _sel(boxes, tier, H, W, patch):
    boxes = np.asarray(boxes, dtype=np.int32).reshape(-1, 4)
    tier = np.asarray(tier, dtype=np.uint8)
    offs = np.asarray([0, len(boxes)], dtype=np.int32)
    return O.select_fine(boxes, tier, offs, 1, H, W, patch)


@pytest.mark.parametrize("patch", [(32, 16), (64, 32, 16)])
def test_no_boxes_gives_coarse_grid(patch):
    H, W = 128, 192
    tok, cu, counts = _sel([], [], H, W, patch)
    rows, cols = H // patch[0], W // patch[0]
    want = [(0, r, c) for r in range(rows) for c in range(cols)]
    assert tok.tolist() == [list(t) for t in want]
    assert cu.tolist() == [0, rows * cols]
    assert counts.tolist() == [[rows * cols] + [0] * (len(patch) - 1)]


@pytest.mark.parametrize("patch", [(32, 16), (64, 32, 16)])
def test_full_frame_box_gives_fine_grid(patch):
    H, W = 128, 192
    top = len(patch) - 1
    tok, cu, counts = _sel([(0, 0, W, H)], [top], H, W, patch)
    rows, cols = H // patch[top], W // patch[top]
    want = [[top, r, c] for r in range(rows) for c in range(cols)]
    assert tok.tolist() == want
    assert counts[0, top] == rows * cols and counts.sum() == rows * cols


def test_tier_zero_box_changes_nothing():
    tok, _, _ = _sel([(0, 0, 128, 128)], [0], 128, 128, (32, 16))
    assert len(tok) == 16 and (tok[:, 0] == 0).all()


def test_mid_tier_stops_at_mid_level():
    tok, _, counts = _sel([(0, 0, 128, 128)], [1], 128, 128, (64, 32, 16))
    assert counts.tolist() == [[0, 16, 0]]


def test_hand_worked_three_level_example():
    # 128x128 frame, patches 64/32/16 -> grids 2x2, 4x4, 8x8.
    # A=(0,0,10,10) tier 2 splits coarse (0,0) and then mid (0,0);
    # B=(70,70,100,100) tier 1 splits coarse (1,1) only; C tier 0 does nothing.
    boxes = [(0, 0, 10, 10), (70, 70, 100, 100), (0, 64, 64, 128)]
    tok, cu, counts = _sel(boxes, [2, 1, 0], 128, 128, (64, 32, 16))
    want = [[0, 0, 1], [0, 1, 0],
            [1, 0, 1], [1, 1, 0], [1, 1, 1], [1, 2, 2], [1, 2, 3], [1, 3, 2], [1, 3, 3],
            [2, 0, 0], [2, 0, 1], [2, 1, 0], [2, 1, 1]]
    assert tok.tolist() == want
    assert counts.tolist() == [[2, 7, 4]]
    assert cu.tolist() == [0, 13]


def test_box_edges_are_half_open():
    # x1 == 32 does not reach the cell that starts at 32; x1 == 33 does.
    tok, _, _ = _sel([(0, 0, 32, 32)], [1], 128, 128, (32, 16))
    assert len(tok) == 16 + 3
    tok, _, _ = _sel([(0, 0, 33, 32)], [1], 128, 128, (32, 16))
    assert len(tok) == 16 + 6
    tok, _, _ = _sel([(31, 31, 33, 33)], [1], 128, 128, (32, 16))
    assert len(tok) == 16 + 12


def test_clipping_and_empty_boxes():
    H = W = 128
    base, _, _ = _sel([], [], H, W, (32, 16))
    for bad in [(-50, -50, 0, 0), (128, 0, 200, 50), (40, 40, 40, 90), (90, 40, 50, 80),
                (0, 200, 128, 300)]:
        tok, _, _ = _sel([bad], [1], H, W, (32, 16))
        assert tok.tolist() == base.tolist(), bad
    # a box hanging over the corner is clipped, not rejected
    tok, _, _ = _sel([(-100, -100, 1, 1)], [1], H, W, (32, 16))
    assert len(tok) == 16 + 3
    tok, _, _ = _sel([(127, 127, 10000, 10000)], [1], H, W, (32, 16))
    assert len(tok) == 16 + 3 and [1, 7, 7] in tok.tolist()


def test_cfg1_token_counts():
    # A 48x48 box covers 2 or 3 coarse cells per axis: T = 16 + 3k, k in {4,6,9}.
    seen = set()
    for x0 in range(0, 81, 4):
        for y0 in range(0, 81, 4):
            tok, _, _ = _sel([(x0, y0, x0 + 48, y0 + 48)], [1], 128, 128, (32, 16))
            kx = (x0 + 47) // 32 - x0 // 32 + 1
            ky = (y0 + 47) // 32 - y0 // 32 + 1
            assert len(tok) == 16 + 3 * kx * ky
            seen.add(len(tok))
    assert seen == {28, 34, 43}
    wl = synth.make_workload(1)
    tok, _, _ = O.select_fine(wl["boxes"], wl["tier"], wl["box_offsets"], 1, 128, 128, (32, 16))
    assert len(tok) in (28, 34, 43)


def _brute_force_pixels(boxes, tier, H, W, patch):
    """Per-pixel definition: paint tier masks, reduce over cell blocks."""
    n = len(patch)
    cover = np.zeros((n + 1, H, W), dtype=bool)    # cover[t]: pixel under a box of tier >= t
    for (x0, y0, x1, y1), t in zip(boxes, tier):
        for yy in range(max(y0, 0), min(y1, H)):
            for xx in range(max(x0, 0), min(x1, W)):
                cover[: int(t) + 1, yy, xx] = True
    level = np.zeros((H, W), dtype=np.int64)
    for l in range(n - 1):
        P = patch[l]
        cell_any = cover[l + 1].reshape(H // P, P, W // P, P).any(axis=(1, 3))
        splits = np.repeat(np.repeat(cell_any, P, axis=0), P, axis=1)
        level = np.where((level == l) & splits, l + 1, level)
    owners = set()
    for yy in range(H):
        for xx in range(W):
            l = int(level[yy, xx])
            owners.add((l, yy // patch[l], xx // patch[l]))
    return sorted(owners), level


@pytest.mark.parametrize("patch", [(16, 8), (32, 16, 8)])
def test_against_per_pixel_brute_force(patch):
    H, W = 64, 96
    rng = np.random.default_rng(11)
    for trial in range(12):
        nb = int(rng.integers(0, 5))
        boxes, tier = [], []
        for _ in range(nb):
            x0, y0 = int(rng.integers(-8, W)), int(rng.integers(-8, H))
            boxes.append((x0, y0, x0 + int(rng.integers(0, 40)), y0 + int(rng.integers(0, 40))))
            tier.append(int(rng.integers(0, len(patch))))
        tok, cu, counts = _sel(boxes, tier, H, W, patch)
        want, level = _brute_force_pixels(boxes, tier, H, W, patch)
        assert [tuple(t) for t in tok.tolist()] == want
        # exact tiling of the frame
        area = sum(patch[l] ** 2 for l, _, _ in tok.tolist())
        assert area == H * W
        # T = N0 + 3 * (number of split cells); split cells counted from the pixel map
        n_split = 0
        for l in range(len(patch) - 1):
            P = patch[l]
            n_split += int((level.reshape(H // P, P, W // P, P).max(axis=(1, 3)) > l).sum())
        assert len(tok) == (H // patch[0]) * (W // patch[0]) + 3 * n_split


def test_batch_is_concatenation_of_frames():
    cfg = synth.config(3)
    wl = synth.make_workload(3)
    tok, cu, counts = O.select_fine(wl["boxes"], wl["tier"], wl["box_offsets"],
                                    cfg.B, cfg.H, cfg.W, cfg.patch)
    assert cu[0] == 0 and (np.diff(cu) == counts.sum(axis=1)).all()
    for i in range(cfg.B):
        lo, hi = wl["box_offsets"][i], wl["box_offsets"][i + 1]
        t1, _, _ = _sel(wl["boxes"][lo:hi], wl["tier"][lo:hi], cfg.H, cfg.W, cfg.patch)
        assert tok[cu[i]:cu[i + 1]].tolist() == t1.tolist()
    # lengths span the range the workload is drawn for (coarse 400 up to ~1000)
    lens = np.diff(cu)
    assert lens.min() >= 400 and lens.max() <= 1600 and len(set(lens.tolist())) > 1


def test_pack_tok_desc():
    tok = np.asarray([[0, 0, 0], [1, 3, 5], [2, 16383, 16383]])
    assert O.pack_tok_desc(tok).tolist() == [0, (1 << 28) | (3 << 14) | 5,
                                             (2 << 28) | (16383 << 14) | 16383]


def test_easy_frames_contribute_no_token():
    # Sec. III-B, A1: an easy frame skips the fine stage.  Hand-worked: three 128x128 frames,
    # patches 32/16 (16 coarse cells); frame 0 has one box inside coarse cell (0, 0) -> 19
    # tokens, frame 1 has a box over the whole frame -> 64, frame 2 has none -> 16.
    boxes = np.asarray([(0, 0, 10, 10), (0, 0, 128, 128)], np.int32)
    tier = np.asarray([1, 1], np.uint8)
    offs = np.asarray([0, 1, 2, 2], np.int32)
    full = O.select_fine(boxes, tier, offs, 3, 128, 128, (32, 16))
    assert full[1].tolist() == [0, 19, 83, 99]
    for hard, want_cu, want_counts in [
            ([1, 1, 1], [0, 19, 83, 99], [[15, 4], [0, 64], [16, 0]]),
            ([1, 0, 1], [0, 19, 19, 35], [[15, 4], [0, 0], [16, 0]]),
            ([0, 1, 0], [0, 0, 64, 64], [[0, 0], [0, 64], [0, 0]]),
            ([0, 0, 0], [0, 0, 0, 0], [[0, 0], [0, 0], [0, 0]])]:
        tok, cu, counts = O.select_fine(boxes, tier, offs, 3, 128, 128, (32, 16),
                                        hard=np.asarray(hard))
        assert cu.tolist() == want_cu and counts.tolist() == want_counts
        # the tokens of the frames that remain are exactly those of the unflagged selection
        keep = np.concatenate([np.arange(full[1][f], full[1][f + 1]) for f in range(3) if hard[f]]
                              or [np.zeros(0, np.int64)]).astype(np.int64)
        assert tok.tolist() == full[0][keep].tolist()
