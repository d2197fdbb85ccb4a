"""The selection through the entry point that allocates nothing (static scratch array, no
context) against cfdetr_select_fine, bit for bit: two calls in a row, the second on a smaller
input, then an overflow and a size beyond the array's limit."""
import ctypes
import sys

import numpy as np
import pytest

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


def _both(K, enc, boxes, tier, offs, B):
    import torch
    b, t, o = enc.upload_boxes(boxes, tier, offs)
    ref = enc.alloc_outputs(B)
    got = enc.alloc_outputs(B)
    for d in (ref, got):
        d["tok_desc"].fill_(-7)
    enc.select_fine(b, t, o, B, ref["tok_desc"], ref["cu_seqlens"], ref["level_counts"])
    enc.sync_status()
    ovf = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    enc.select_fine_static(b, t, o, B, got["tok_desc"], got["cu_seqlens"], got["level_counts"], ovf)
    torch.cuda.synchronize()
    return ref, got, int(ovf.item())


def test_static_selection_equals_the_context_one(K):
    cfg = synth.config(5)                           # three levels, 12 frames of 1024 x 1024
    _, boxes, tier, offs, _ = synth.make_frames(cfg, 5)
    w = synth.make_weights(synth.replace(cfg, layers=1), 1)
    enc = K.Encoder(synth.replace(cfg, layers=1), w)
    _say("[case] static selection, 12 frames")
    ref, got, ovf = _both(K, enc, boxes, tier, offs, cfg.B)
    assert ovf == 0
    for k in ("tok_desc", "cu_seqlens", "level_counts"):
        np.testing.assert_array_equal(got[k].cpu().numpy(), ref[k].cpu().numpy())
    assert int(ref["cu_seqlens"][-1]) > cfg.B * cfg.n_cells(0)      # something was refined
    # second call, smaller input: the first 5 frames, and only every other box of them
    B2 = 5
    keep = np.concatenate([np.arange(offs[f], offs[f + 1])[::2] for f in range(B2)]).astype(np.int64)
    offs2 = np.concatenate([[0], np.cumsum([len(np.arange(offs[f], offs[f + 1])[::2])
                                            for f in range(B2)])]).astype(np.int32)
    _say("[case] static selection, second call with 5 frames and half of their boxes")
    ref2, got2, ovf2 = _both(K, enc, boxes[keep], tier[keep], offs2, B2)
    assert ovf2 == 0
    for k in ("tok_desc", "cu_seqlens", "level_counts"):
        np.testing.assert_array_equal(got2[k].cpu().numpy(), ref2[k].cpu().numpy())
    assert int(ref2["cu_seqlens"][-1]) < int(ref["cu_seqlens"][5])  # fewer tokens than before
    # a third call without any box: flags of the earlier calls must be gone
    none = np.zeros((0, 4), np.int32)
    ref3, got3, _ = _both(K, enc, none, np.zeros(0, np.uint8), np.zeros(B2 + 1, np.int32), B2)
    assert got3["cu_seqlens"].cpu().tolist() == [f * cfg.n_cells(0) for f in range(B2 + 1)]
    np.testing.assert_array_equal(got3["tok_desc"].cpu().numpy(), ref3["tok_desc"].cpu().numpy())
    enc.close()


def test_static_selection_reports_overflow_and_rejects_sizes_beyond_its_array(K):
    import torch
    cfg = synth.Config("ovf", 2, 128, 128, (32, 16), 64, 2, 1, 128, "f32")
    enc = K.Encoder(cfg, synth.make_weights(cfg, 3), max_tokens_total=40)
    boxes = np.asarray([[0, 0, 128, 128]], np.int32)      # frame 1 alone needs 64 tokens
    b, t, o = enc.upload_boxes(boxes, np.asarray([1], np.uint8), np.asarray([0, 0, 1], np.int32))
    out = enc.alloc_outputs(cfg.B)
    out["tok_desc"].fill_(-7)
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda")
    _say("[case] static selection, overflow")
    enc.select_fine_static(b, t, o, cfg.B, out["tok_desc"], out["cu_seqlens"], out["level_counts"], ovf)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 1
    assert out["cu_seqlens"].cpu().tolist() == [0, 0, 0]
    assert (out["tok_desc"].cpu().numpy() == -7).all()
    enc.close()
    # 64 frames of 4096 x 4096 at patches 16 / 8: 64 * 65536 flag bytes > 1 MiB: refused on the host
    big = K.CfdetrConfig()
    big.n_levels = 2
    big.patch[0], big.patch[1], big.patch[2] = 16, 8, 0
    big.img_h = big.img_w = 4096
    big.d_model, big.n_heads, big.n_layers, big.d_ffn = 64, 2, 1, 128
    big.max_batch, big.max_tokens_total = 64, 64 * 65536
    big.image_dtype, big.act_dtype, big.ln_eps = K.CFDETR_FP32, K.CFDETR_BF16, 1e-5
    _say("[case] static selection, size beyond the array")
    with pytest.raises(K.CfdetrError) as ei:
        K.cfdetr_select_fine_static(big, b.data_ptr(), t.data_ptr(), o.data_ptr(), 64,
                                    out["tok_desc"].data_ptr(), out["cu_seqlens"].data_ptr(), None,
                                    ovf.data_ptr(), 0)
    assert ei.value.status == K.CFDETR_ECAPACITY
    assert "static scratch" in str(ei.value)
