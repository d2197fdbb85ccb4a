"""Pins for the oracle's A1 difficulty test and A2 region proposal (Sec. III-B).

Checked against things other than the oracle itself: a hand-worked example stored as
text (tests/golden/roi_worked_example.txt), the limiting cases the definition fixes,
and a brute force over pixel squares for the rounding of a region's edges.
"""
import os

import numpy as np
import pytest

from oracle import cfdetr_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "roi_worked_example.txt")
BOXES = [(0.50, 0.50, 0.20, 0.40), (0.25, 0.50, 0.10, 0.20), (0.90, 0.10, 0.30, 0.30),
         (0.10, 0.90, 0.05, 0.05), (0.70, 0.70, 0.10, 0.10), (0.40, 0.20, 0.10, 0.10)]


def _golden():
    out = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            case = out.setdefault(p[0], {"boxes": []})
            if p[1] == "hard":
                case["hard"], case["mean"] = int(p[2]), float(p[4])
            else:
                case["boxes"].append([int(v) for v in p[2:6]])
    return out


def _queries(conf, boxes=BOXES):
    q = np.zeros((1, len(conf), 5))
    q[0, :, :4] = np.asarray(boxes[:len(conf)])
    q[0, :, 4] = conf
    return q


@pytest.mark.parametrize("case,conf,thr", [
    ("A", [0.95, 0.5, 0.3, 0.01, 0.02, 0.0], (0.8, 0.05)),
    ("B", [0.95, 0.07, 0.06, 0.01, 0.02, 0.0], (0.8, 0.05)),
    ("C", [0.75, 0.0625, 0.5, 0.0], (0.75, 0.0625)),
    ("D1", [0.125, 0.0, 0.0, 0.0], (0.75, 0.0625)),
    ("D2", [0.25, 0.0, 0.0, 0.0], (0.75, 0.0625)),
])
def test_hand_worked_example(case, conf, thr):
    g = _golden()[case]
    boxes, tier, offs, hard, mean = O.propose_rois(_queries(conf), 100, 200, thr[0], thr[1], tier=1)
    assert hard.tolist() == [g["hard"]]
    assert mean[0] == pytest.approx(g["mean"], abs=1e-12)
    assert boxes.tolist() == g["boxes"]
    assert offs.tolist() == [0, len(g["boxes"])]
    assert tier.tolist() == [1] * len(g["boxes"])


def test_limits_of_the_difficulty_test():
    # every query certain: nothing is left to average -> easy
    assert O.frame_hardness([0.9, 0.99, 0.81], 0.8, 0.05) == (False, 0.0)
    # all background -> easy; all intermediate -> hard
    assert O.frame_hardness([0.01] * 50, 0.8, 0.05)[0] is False
    assert O.frame_hardness([0.4] * 50, 0.8, 0.05)[0] is True
    # the certain queries do not enter the average, however many there are
    hard, mean = O.frame_hardness([0.9] * 100 + [0.06, 0.06], 0.8, 0.05)
    assert hard is True and mean == pytest.approx(0.06)
    # adding background queries dilutes the average: hard -> easy
    assert O.frame_hardness([0.5] + [0.0] * 5, 0.8, 0.05)[0] is True
    assert O.frame_hardness([0.5] + [0.0] * 50, 0.8, 0.05)[0] is False


def test_region_covers_exactly_the_pixels_the_box_touches():
    """Brute force over unit pixel squares: pixel (px, py) belongs to the region iff its
    open square (px, px+1) x (py, py+1) meets the open real-valued box."""
    rng = np.random.default_rng(5)
    H, W = 37, 53
    for _ in range(300):
        cx, cy = rng.uniform(-0.1, 1.1, 2)
        w, h = rng.uniform(0.01, 0.6, 2)
        scale = rng.choice([1.0, 1.5])
        x0, y0, x1, y1 = O.roi_box(cx, cy, w, h, H, W, scale)
        lo_x, hi_x = cx * W - 0.5 * scale * w * W, cx * W + 0.5 * scale * w * W
        lo_y, hi_y = cy * H - 0.5 * scale * h * H, cy * H + 0.5 * scale * h * H
        inside = np.zeros((H, W), bool)
        for py in range(H):
            for px in range(W):
                inside[py, px] = (px + 1 > lo_x and px < hi_x and py + 1 > lo_y and py < hi_y)
        want = np.zeros((H, W), bool)
        want[y0:y1, x0:x1] = True
        assert (inside == want).all()


def test_min_side_and_scale():
    # a 4-pixel box grown to at least 32 pixels about its centre
    assert O.roi_box(0.5, 0.5, 0.02, 0.04, 100, 200, 1.0, 32.0) == (84, 34, 116, 66)
    # scale 2 doubles the side about the centre
    assert O.roi_box(0.5, 0.5, 0.1, 0.1, 100, 200, 2.0) == (80, 40, 120, 60)
    # integer edges stay where they are (no outward step)
    assert O.roi_box(0.25, 0.5, 0.1, 0.2, 100, 200) == (40, 40, 60, 60)


def test_batch_is_the_concatenation_of_its_frames():
    rng = np.random.default_rng(11)
    q = rng.uniform(0, 1, (5, 40, 5))
    q[..., 4] = rng.choice([0.001, 0.02, 0.3, 0.7, 0.9], (5, 40), p=[0.5, 0.3, 0.1, 0.05, 0.05])
    q[3, :, 4] = 0.001     # an easy frame in the middle
    boxes, tier, offs, hard, mean = O.propose_rois(q, 96, 128, 0.8, 0.05, tier=2)
    assert hard[3] == 0 and offs[4] == offs[3]
    parts = [O.propose_rois(q[f:f + 1], 96, 128, 0.8, 0.05, tier=2) for f in range(5)]
    assert np.array_equal(boxes, np.concatenate([p[0] for p in parts]))
    assert offs.tolist() == [0] + np.cumsum([len(p[0]) for p in parts]).tolist()
    assert hard.tolist() == [int(p[3][0]) for p in parts]
    # the proposals drive the selection: an easy frame keeps its coarse grid
    tok, cu, counts = O.select_fine(boxes, tier, offs, 5, 96, 128, (32, 16, 8))
    assert counts[3].tolist() == [12, 0, 0]


# ------------------------------------------------------------------ merge of the two stages
def _merge_fixture():
    path = os.path.join(os.path.dirname(__file__), "golden", "merge_worked_example.txt")
    coarse, fine, out = [], [], {}
    for line in open(path):
        p = line.split()
        if not p or p[0] == "#":
            continue
        if p[0] == "in":
            (coarse if p[1] == "coarse" else fine).append([float(v) for v in p[2:]])
        elif p[2] == "count":
            out.setdefault(int(p[1]), {"count": int(p[3]), "det": []})
        else:
            out[int(p[1])]["det"].append((int(p[3]), [float(v) for v in p[4:]]))
    return np.array(coarse, np.float32), np.array(fine, np.float32), out


def test_merge_matches_the_hand_worked_example():
    coarse, fine, want = _merge_fixture()
    c = np.stack([coarse, coarse])
    f = np.stack([fine, fine])
    det, src, count = O.merge_detections(c, f, np.array([1, 0]), 0.75, 0.25)
    for frame, w in want.items():
        assert count[frame] == w["count"]
        for i, (s, row) in enumerate(w["det"]):
            assert src[frame, i] == s
            np.testing.assert_array_equal(det[frame, i], np.array(row, np.float32))
        assert (src[frame, w["count"]:] == 255).all() and not det[frame, w["count"]:].any()


def test_merge_counts_order_and_limits():
    rng = np.random.default_rng(5)
    B, Q = 5, 37
    c = rng.uniform(0, 1, (B, Q, 5)).astype(np.float32)
    f = rng.uniform(0, 1, (B, Q, 5)).astype(np.float32)
    hard = np.array([1, 0, 1, 1, 0])
    det, src, count = O.merge_detections(c, f, hard, 0.8, 0.3)
    for b in range(B):
        n_c = int((c[b, :, 4] > np.float32(0.8)).sum())
        n_f = int((f[b, :, 4] > np.float32(0.3)).sum()) if hard[b] else 0
        assert count[b] == n_c + n_f                                   # closed form of the count
        assert (src[b, :n_c] == 0).all() and (src[b, n_c:n_c + n_f] == 1).all()
        # the kept rows are the stage's rows in query order: confidences form the same sequence
        np.testing.assert_array_equal(det[b, :n_c, 4], c[b, c[b, :, 4] > np.float32(0.8), 4])
        if hard[b]:
            np.testing.assert_array_equal(det[b, n_c:n_c + n_f], f[b, f[b, :, 4] > np.float32(0.3)])
    # limits: nothing is certain and nothing refined -> empty; everything passes -> both stages whole
    det, src, count = O.merge_detections(c, f, hard, 1.0, 1.0)
    assert not count.any() and not det.any() and (src == 255).all()
    det, src, count = O.merge_detections(c, f, np.ones(B, int), -1.0, -1.0)
    assert (count == 2 * Q).all()
    np.testing.assert_array_equal(det[:, :Q], c)
    np.testing.assert_array_equal(det[:, Q:], f)
    # an easy frame never shows a fine-stage row, whatever the fine stage holds
    det, src, count = O.merge_detections(c, np.full_like(f, 0.99), np.zeros(B, int), 0.8, 0.0)
    assert not (src == 1).any()
