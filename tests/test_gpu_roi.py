"""GPU parity of the A1 difficulty test and A2 region proposal (Sec. III-B) against the
CPU oracle: boxes, refinement levels, offsets and easy/hard flags bit-exact, the average
confidence within 1e-6."""
import sys

import numpy as np
import pytest

from oracle import cfdetr_oracle as O
from paper_2505_23317_amd import synth

pytestmark = pytest.mark.gpu

TAU_HI, TAU_LO = float(np.float32(0.8)), float(np.float32(0.05))


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def K():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_23317_amd import cfdetr
    cfdetr.load_library()
    return cfdetr


def _ctx(K, cfg):
    one = synth.replace(cfg, layers=1)
    return K.Encoder(one, synth.make_weights(one, 1))


def gpu_propose(K, enc, q, tau_hi, tau_lo, tier, scale=1.0, min_side=0.0, max_boxes=None):
    import torch
    B, Q = q.shape[:2]
    cap = B * Q if max_boxes is None else max_boxes
    dq = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
    boxes = torch.full((max(cap, 1), 4), -7, dtype=torch.int32, device="cuda")
    t = torch.full((max(cap, 1),), 255, dtype=torch.uint8, device="cuda")
    offs = torch.full((B + 1,), -1, dtype=torch.int32, device="cuda")
    hard = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    mean = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
    p = K.CfdetrRoiParams(tau_hi, tau_lo, scale, min_side, tier)
    K.cfdetr_propose_rois(enc.ctx, dq.data_ptr(), B, Q, p, cap, boxes.data_ptr(), t.data_ptr(),
                          offs.data_ptr(), hard.data_ptr(), mean.data_ptr(), 0)
    torch.cuda.synchronize()
    return boxes, t, offs, hard, mean


def check(K, enc, cfg, q, tier, scale=1.0, min_side=0.0, tau=(TAU_HI, TAU_LO), label=""):
    got = gpu_propose(K, enc, q, tau[0], tau[1], tier, scale, min_side)
    rb, rt, ro, rh, rm = O.propose_rois(q.astype(np.float32), cfg.H, cfg.W, tau[0], tau[1], tier,
                                        float(np.float32(scale)), float(np.float32(min_side)))
    n = int(ro[-1])
    np.testing.assert_array_equal(got[2].cpu().numpy(), ro)
    np.testing.assert_array_equal(got[3].cpu().numpy(), rh)
    np.testing.assert_array_equal(got[0].cpu().numpy()[:n], rb)
    np.testing.assert_array_equal(got[1].cpu().numpy()[:n], rt)
    assert (got[0].cpu().numpy()[n:] == -7).all()      # nothing written past the total
    assert np.abs(got[4].cpu().numpy().astype(np.float64) - rm).max() <= 1e-6
    _say(f"[roi] {label}: B={q.shape[0]} Q={q.shape[1]} regions={n} hard={rh.tolist()}")
    return got, (rb, rt, ro, rh, rm)


@pytest.mark.parametrize("cfg_id,Q", [(3, 128), (3, 900), (5, 300), (4, 1000)])
def test_region_proposal_matches_the_oracle(K, cfg_id, Q):
    cfg = synth.config(cfg_id)
    enc = _ctx(K, cfg)
    q = synth.make_queries(cfg, seed=cfg_id, n_queries=Q, easy_frames=(1,))
    (_, _, ro, rh, _) = check(K, enc, cfg, q, cfg.n_levels - 1, label=f"cfg{cfg_id}")[1]
    assert rh[1] == 0 and ro[2] == ro[1]            # the easy frame proposes nothing
    check(K, enc, cfg, q, 1, scale=1.5, min_side=32.0, label=f"cfg{cfg_id} scaled")
    enc.close()


def test_threshold_edges_and_degenerate_batches(K):
    cfg = synth.config(2)
    enc = _ctx(K, cfg)
    box = [0.5, 0.5, 0.2, 0.4]
    # exact binary thresholds: equal to tau_hi stays intermediate, equal to tau_lo is background;
    # an average exactly at tau_lo is hard
    for conf in ([0.75, 0.0625, 0.5, 0.0], [0.125, 0.0, 0.0, 0.0], [0.25, 0.0, 0.0, 0.0],
                 [0.9, 0.99], [0.0], [1.0], [0.7]):
        q = np.zeros((1, len(conf), 5), np.float32)
        q[0, :, :4] = box
        q[0, :, 4] = conf
        check(K, enc, cfg, q, 1, tau=(0.75, 0.0625), label=f"conf {conf}")
    # boxes hanging over every edge of the frame, and far outside it
    q = np.zeros((1, 6, 5), np.float32)
    q[0, :, 4] = 0.5
    q[0, :, :4] = [[0.0, 0.0, 0.3, 0.3], [1.0, 1.0, 0.3, 0.3], [0.5, -0.2, 0.1, 0.1],
                   [3.0, 3.0, 0.1, 0.1], [0.5, 0.5, 5.0, 5.0], [0.5, 0.5, 0.0, 0.0]]
    check(K, enc, cfg, q, 1, tau=(0.75, 0.0625), label="edges")
    enc.close()


def test_region_overflow_is_reported_not_truncated(K):
    import torch
    cfg = synth.config(3)
    enc = _ctx(K, cfg)
    q = synth.make_queries(cfg, seed=9, n_queries=128)
    total = int(O.propose_rois(q, cfg.H, cfg.W, TAU_HI, TAU_LO, 1)[2][-1])
    boxes, t, offs, hard, mean = gpu_propose(K, enc, q, TAU_HI, TAU_LO, 1, max_boxes=total - 1)
    assert offs.cpu().numpy().tolist() == [0] * (cfg.B + 1)
    assert (boxes.cpu().numpy() == -7).all()
    with pytest.raises(K.CfdetrError) as e:
        enc.sync_status()
    assert e.value.status == K.CFDETR_ECAPACITY
    # exactly enough room is fine
    enc2 = _ctx(K, cfg)
    got = gpu_propose(K, enc2, q, TAU_HI, TAU_LO, 1, max_boxes=total)
    assert int(got[2].cpu().numpy()[-1]) == total
    enc2.sync_status()
    enc.close()
    enc2.close()


def test_host_side_argument_errors_of_the_proposal(K):
    import torch
    cfg = synth.config(2)
    enc = _ctx(K, cfg)
    q = torch.zeros((1, 8, 5), dtype=torch.float32, device="cuda")
    out = [torch.zeros(64, dtype=torch.int32, device="cuda") for _ in range(5)]
    ok = K.CfdetrRoiParams(0.8, 0.05, 1.0, 0.0, 1)

    def call(params=ok, B=1, Q=8, qp=None, cap=8):
        K.cfdetr_propose_rois(enc.ctx, q.data_ptr() if qp is None else qp, B, Q, params, cap,
                              out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(),
                              out[3].data_ptr(), out[4].data_ptr(), 0)

    call()
    for bad in (K.CfdetrRoiParams(0.05, 0.8, 1.0, 0.0, 1), K.CfdetrRoiParams(0.8, 0.05, -1.0, 0.0, 1),
                K.CfdetrRoiParams(0.8, 0.05, 1.0, -2.0, 1), K.CfdetrRoiParams(0.8, 0.05, 1.0, 0.0, 2),
                K.CfdetrRoiParams(float("nan"), 0.05, 1.0, 0.0, 1)):
        with pytest.raises(K.CfdetrError) as e:
            call(params=bad)
        assert e.value.status == K.CFDETR_EINVAL
    for kw in (dict(Q=0), dict(qp=0), dict(qp=q.data_ptr() + 4), dict(cap=-1)):
        with pytest.raises(K.CfdetrError) as e:
            call(**kw)
        assert e.value.status == K.CFDETR_EINVAL
    with pytest.raises(K.CfdetrError) as e:
        call(B=2)
    assert e.value.status == K.CFDETR_ECAPACITY
    torch.cuda.synchronize()
    enc.close()


def test_proposal_feeds_the_selection_on_the_device(K):
    """Queries -> regions -> token table without the boxes leaving the device."""
    import torch
    cfg = synth.config(5)
    enc = _ctx(K, cfg)
    q = synth.make_queries(cfg, seed=21, n_queries=200, easy_frames=(0, 7))
    boxes, t, offs, hard, mean = gpu_propose(K, enc, q, TAU_HI, TAU_LO, 2)
    out = enc.alloc_outputs(cfg.B)
    enc.select_fine(boxes, t, offs, cfg.B, out["tok_desc"], out["cu_seqlens"], out["level_counts"])
    enc.sync_status()
    torch.cuda.synchronize()
    rb, rt, ro, rh, rm = O.propose_rois(q, cfg.H, cfg.W, TAU_HI, TAU_LO, 2)
    tok, cu, counts = O.select_fine(rb, rt, ro, cfg.B, cfg.H, cfg.W, cfg.patch)
    np.testing.assert_array_equal(out["cu_seqlens"].cpu().numpy(), cu)
    np.testing.assert_array_equal(out["level_counts"].cpu().numpy(), counts)
    np.testing.assert_array_equal(out["tok_desc"].cpu().numpy()[:cu[-1]], O.pack_tok_desc(tok))
    n0 = cfg.n_cells(0)
    assert counts[0].tolist() == [n0, 0, 0] and counts[7].tolist() == [n0, 0, 0]
    enc.close()


# ------------------------------------------------------------------ merge of the two stages
def gpu_merge(K, enc, coarse, fine, hard, tau_hi, tau_fine):
    import torch
    B, Q = coarse.shape[:2]
    dc = torch.from_numpy(np.ascontiguousarray(coarse, dtype=np.float32)).cuda()
    df = torch.from_numpy(np.ascontiguousarray(fine, dtype=np.float32)).cuda()
    dh = torch.from_numpy(np.ascontiguousarray(hard, dtype=np.int32)).cuda()
    det = torch.full((B, 2 * Q, 5), -7.0, dtype=torch.float32, device="cuda")
    src = torch.full((B, 2 * Q), 9, dtype=torch.uint8, device="cuda")
    count = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    enc.merge_detections(dc, df, dh, tau_hi, tau_fine, det, src, count)
    enc.sync_status()
    torch.cuda.synchronize()
    return det.cpu().numpy(), src.cpu().numpy(), count.cpu().numpy()


@pytest.mark.parametrize("Q", [8, 63, 128, 300, 1000])
def test_merge_of_the_two_stages_is_bit_exact(K, Q):
    cfg = synth.replace(synth.config(3), B=6)
    enc = _ctx(K, cfg)
    _say(f"[case] merge Q={Q}")
    coarse = synth.make_queries(cfg, seed=11, n_queries=Q, easy_frames=(2,))
    fine = synth.make_queries(cfg, seed=12, n_queries=Q)
    hard = O.propose_rois(coarse, cfg.H, cfg.W, TAU_HI, TAU_LO, 1)[3]
    for tau_hi, tau_fine in ((TAU_HI, 0.3), (TAU_HI, TAU_LO), (0.0, 0.0), (1.0, 1.0), (-1.0, -1.0)):
        got = gpu_merge(K, enc, coarse, fine, hard, tau_hi, tau_fine)
        ref = O.merge_detections(coarse, fine, hard, float(np.float32(tau_hi)),
                                 float(np.float32(tau_fine)))
        np.testing.assert_array_equal(got[2], ref[2])
        np.testing.assert_array_equal(got[1], ref[1])
        np.testing.assert_array_equal(got[0], ref[0])
    # thresholds that are exact binary fractions: equality keeps nothing
    c2 = coarse.copy()
    c2[:, ::2, 4] = 0.75
    f2 = fine.copy()
    f2[:, ::3, 4] = 0.25
    got = gpu_merge(K, enc, c2, f2, np.ones(cfg.B, np.int32), 0.75, 0.25)
    ref = O.merge_detections(c2, f2, np.ones(cfg.B, np.int32), 0.75, 0.25)
    for g, r in zip(got, ref):
        np.testing.assert_array_equal(g, r)
    # a single query per frame
    c1, f1 = coarse[:, :1].copy(), fine[:, :1].copy()
    c1[:, 0, 4] = [0.9, 0.1, 0.9, 0.1, 0.9, 0.1]
    f1[:, 0, 4] = [0.9, 0.9, 0.1, 0.1, 0.9, 0.9]
    h1 = np.array([1, 1, 1, 1, 0, 0], np.int32)
    got = gpu_merge(K, enc, c1, f1, h1, TAU_HI, 0.3)
    ref = O.merge_detections(c1, f1, h1, TAU_HI, float(np.float32(0.3)))
    assert ref[2].tolist() == [2, 1, 1, 0, 1, 0]
    for g, r in zip(got, ref):
        np.testing.assert_array_equal(g, r)
    enc.close()


def test_merge_argument_errors(K):
    import torch
    cfg = synth.config(2)
    enc = _ctx(K, cfg)
    q = torch.zeros((1, 8, 5), dtype=torch.float32, device="cuda")
    hard = torch.zeros(1, dtype=torch.int32, device="cuda")
    det = torch.zeros((1, 16, 5), dtype=torch.float32, device="cuda")
    src = torch.zeros((1, 16), dtype=torch.uint8, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")

    def call(B=1, Q=8, tau=0.8, coarse=q.data_ptr()):
        K.cfdetr_merge_detections(enc.ctx, coarse, q.data_ptr(), hard.data_ptr(), B, Q, tau, 0.3,
                                  det.data_ptr(), src.data_ptr(), cnt.data_ptr(), 0)

    call()
    for kw, status in ((dict(B=0), K.CFDETR_EINVAL), (dict(B=2), K.CFDETR_ECAPACITY),
                       (dict(Q=0), K.CFDETR_EINVAL), (dict(tau=float("nan")), K.CFDETR_EINVAL),
                       (dict(coarse=None), K.CFDETR_EINVAL)):
        with pytest.raises(K.CfdetrError) as e:
            call(**kw)
        assert e.value.status == status, kw
    enc.close()
