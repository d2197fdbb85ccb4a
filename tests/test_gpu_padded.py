"""The fine pass in the paper's padded form (Sec. III-B, A3: token sets brought to one
length) against the variable-length form and the CPU oracle: every real token gets the
same result, bit for bit, as without padding."""
import sys

import numpy as np
import pytest

from oracle import cfdetr_oracle as O
from paper_2505_23317_amd import synth

pytestmark = pytest.mark.gpu


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


def run_both(K, cfg, wl, act, t_pad=None, extra=0):
    import torch
    enc = K.Encoder(cfg, wl["weights"], act_dtype=act)
    img = enc.upload_images(wl["images"])
    b, t, o = enc.upload_boxes(wl["boxes"], wl["tier"], wl["box_offsets"])
    out = enc.alloc_outputs(cfg.B)
    enc.coarse_encode(img, cfg.B, out["x0_cache"], out["y_coarse"])
    enc.select_fine(b, t, o, cfg.B, out["tok_desc"], out["cu_seqlens"], out["level_counts"])
    enc.fine_encode(img, cfg.B, out["tok_desc"], out["cu_seqlens"], out["x0_cache"], out["y_mixed"])
    torch.cuda.synchronize()
    cu = out["cu_seqlens"].cpu().numpy()
    longest = int(np.diff(cu).max())
    tp = (longest + extra) if t_pad is None else t_pad
    y_pad = torch.zeros((cfg.B * tp, cfg.d), dtype=torch.float32, device="cuda")
    enc.fine_encode_padded(img, cfg.B, out["tok_desc"], out["cu_seqlens"], out["x0_cache"], tp, y_pad)
    torch.cuda.synchronize()
    return enc, cu, tp, out["y_mixed"].cpu().numpy(), y_pad.cpu().numpy()


@pytest.mark.parametrize("act", ["bf16", "fp32"])
@pytest.mark.parametrize("extra", [0, 37])
def test_padded_form_gives_every_real_token_the_same_result(K, act, extra):
    cfg = synth.replace(synth.config(3), layers=2)
    wl = synth.make_workload(cfg, seed=61)
    enc, cu, tp, y_var, y_pad = run_both(K, cfg, wl, act, extra=extra)
    enc.sync_status()
    for f in range(cfg.B):
        n = cu[f + 1] - cu[f]
        np.testing.assert_array_equal(y_pad[f * tp:f * tp + n], y_var[cu[f]:cu[f + 1]])
    assert np.isfinite(y_pad).all()
    _say(f"[padded] {act}: lengths {np.diff(cu).tolist()} padded to {tp}")
    enc.close()


def test_padded_form_against_the_oracle(K):
    cfg = synth.replace(synth.config(1), B=3, layers=2)
    wl = synth.make_workload(cfg, seed=5)
    enc, cu, tp, y_var, y_pad = run_both(K, cfg, wl, "fp32", extra=3)
    enc.sync_status()
    tok, cu_o, _ = O.select_fine(wl["boxes"], wl["tier"], wl["box_offsets"], cfg.B, cfg.H, cfg.W,
                                 cfg.patch)
    xs = [O.embed_frame(wl["images"][f], tok[cu_o[f]:cu_o[f + 1]], cfg.patch, wl["weights"])
          for f in range(cfg.B)]
    ref = O.encode_padded(xs, wl["weights"], cfg.heads)
    for f in range(cfg.B):
        n = cu[f + 1] - cu[f]
        err = np.abs(y_pad[f * tp:f * tp + n] - ref[f]).max() / np.abs(ref[f]).max()
        assert err <= 1e-4, (f, err)
    enc.close()


def test_padded_form_errors(K):
    import torch
    cfg = synth.replace(synth.config(3), layers=1)
    wl = synth.make_workload(cfg, seed=61)
    # a pad length below the longest frame is reported, not silently accepted
    enc, cu, tp, y_var, y_pad = run_both(K, cfg, wl, "bf16", t_pad=int(np.diff(
        O.select_fine(wl["boxes"], wl["tier"], wl["box_offsets"], cfg.B, cfg.H, cfg.W,
                      cfg.patch)[1]).max()) - 1)
    with pytest.raises(K.CfdetrError) as e:
        enc.sync_status()
    assert e.value.status == K.CFDETR_ECAPACITY
    enc.close()
    enc = K.Encoder(cfg, wl["weights"])
    img = enc.upload_images(wl["images"])
    out = enc.alloc_outputs(cfg.B)
    y = torch.zeros((enc.max_tokens, cfg.d), dtype=torch.float32, device="cuda")
    with pytest.raises(K.CfdetrError) as e:      # below the coarse grid
        enc.fine_encode_padded(img, cfg.B, out["tok_desc"], out["cu_seqlens"], None, cfg.n_cells(0) - 1, y)
    assert e.value.status == K.CFDETR_EINVAL
    with pytest.raises(K.CfdetrError) as e:      # does not fit the work space
        enc.fine_encode_padded(img, cfg.B, out["tok_desc"], out["cu_seqlens"], None,
                               enc.max_tokens // cfg.B + 1, y)
    assert e.value.status == K.CFDETR_ECAPACITY
    enc.close()


def test_padded_form_reports_a_frame_without_tokens(K):
    """A frame that skipped the fine stage has no token; the padded form has no place for an
    empty frame (all of its keys would be masked): reported, and every row stays finite."""
    import torch
    cfg = synth.replace(synth.config(3), B=3, H=320, W=320, layers=1)
    wl = synth.make_workload(cfg, seed=63)
    enc = K.Encoder(cfg, wl["weights"], act_dtype="bf16")
    img = enc.upload_images(wl["images"])
    b, t, o = enc.upload_boxes(wl["boxes"], wl["tier"], wl["box_offsets"])
    out = enc.alloc_outputs(cfg.B)
    hard = torch.tensor([1, 0, 1], dtype=torch.int32, device="cuda")
    enc.select_fine_hard(b, t, o, hard, cfg.B, out["tok_desc"], out["cu_seqlens"], None)
    enc.sync_status()
    cu = out["cu_seqlens"].cpu().numpy()
    assert cu[2] == cu[1]
    tp = int(np.diff(cu).max())
    y = torch.zeros((cfg.B * tp, cfg.d), dtype=torch.float32, device="cuda")
    _say(f"[case] padded form with an empty frame, lengths {np.diff(cu).tolist()} padded to {tp}")
    enc.fine_encode_padded(img, cfg.B, out["tok_desc"], out["cu_seqlens"], None, tp, y)
    with pytest.raises(K.CfdetrError) as e:
        enc.sync_status()
    assert e.value.status == K.CFDETR_ECAPACITY
    assert np.isfinite(y.cpu().numpy()).all()
    enc.close()
