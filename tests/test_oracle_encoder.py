"""Pins for the oracle's token embedding and encoder (Sec. II-A; A1-A3, Sec. III-B).

The oracle is checked against closed forms, textbook special cases, pure-Python
brute force on tiny inputs and stock library layers in float64 (torch's conv2d,
LayerNorm, GELU, MultiheadAttention and pre-LN TransformerEncoder), and against
the invariants the method's definition fixes: no RoI -> the coarse encoder,
RoI everywhere -> a plain fine-patch ViT encoder, batched == frame by frame,
padded+masked == variable length.
"""
import math

import numpy as np
import pytest
import torch

from oracle import cfdetr_oracle as O
from paper_2505_23317_amd import synth


def _wl(cfg, seed=5, sharp=False):
    return synth.make_workload(cfg, seed=seed, sharp=sharp)


# ----------------------------------------------------------------- positions
def test_pos_encoding_closed_form():
    # d=8 -> D=4, two frequencies: 1 and 10000^(-1/2) = 0.01
    H, W, P = 64, 128, 16
    pe = O.pos_encoding(P, 0, 1, H, W, 8)       # v = 8/64 = 1/8, u = 24/128 = 3/16
    want = [math.sin(math.pi / 4), math.cos(math.pi / 4),
            math.sin(2 * math.pi * 0.125 * 0.01), math.cos(2 * math.pi * 0.125 * 0.01),
            math.sin(2 * math.pi * 3 / 16), math.cos(2 * math.pi * 3 / 16),
            math.sin(2 * math.pi * 3 / 16 * 0.01), math.cos(2 * math.pi * 3 / 16 * 0.01)]
    np.testing.assert_allclose(pe, want, rtol=0, atol=1e-15)
    assert abs(pe[0] - math.sqrt(0.5)) < 1e-15


def test_pos_encoding_pairs_and_scale_invariance():
    pe = O.pos_encoding(16, 5, 9, 256, 320, 64)
    np.testing.assert_allclose(pe[0::2] ** 2 + pe[1::2] ** 2, 1.0, atol=1e-14)
    # normalised coordinates: the same relative centre gives the same vector
    np.testing.assert_allclose(pe, O.pos_encoding(32, 5, 9, 512, 640, 64), atol=1e-15)
    # a coarse cell's centre is the shared corner of its four children: the mean of the
    # children's (u,v) equals the parent's, so the lowest-frequency terms nearly agree
    # while the vectors themselves differ (levels do not alias)
    kids = [O.pos_encoding(8, 10 + a, 18 + b, 256, 320, 64) for a in (0, 1) for b in (0, 1)]
    assert np.abs(np.mean(kids, axis=0) - pe).max() < 2e-2
    assert np.abs(kids[0] - pe).max() > 1e-3
    # transposing the frame swaps the two halves
    a = O.pos_encoding(16, 2, 7, 128, 128, 32)
    b = O.pos_encoding(16, 7, 2, 128, 128, 32)
    np.testing.assert_allclose(a[:16], b[16:], atol=0)
    np.testing.assert_allclose(a[16:], b[:16], atol=0)


# ----------------------------------------------------------------- embedding
def test_embed_matches_strided_conv(tiny_cfg):
    cfg = tiny_cfg
    wl = _wl(cfg)
    w = wl["weights"]
    img = wl["images"][0]
    for lvl, P in enumerate(cfg.patch):
        rows, cols = cfg.grid(lvl)
        tok = np.asarray([(lvl, r, c) for r in range(rows) for c in range(cols)])
        got = O.embed_frame(img, tok, cfg.patch, w)
        conv = torch.nn.functional.conv2d(
            torch.from_numpy(img).double()[None],
            torch.from_numpy(w[f"w_embed{lvl}"]).double().reshape(cfg.d, 3, P, P),
            torch.from_numpy(w[f"b_embed{lvl}"]).double(), stride=P)[0]      # [d, rows, cols]
        want = conv.permute(1, 2, 0).reshape(rows * cols, cfg.d).numpy()
        pe = np.stack([O.pos_encoding(P, r, c, cfg.H, cfg.W, cfg.d)
                       for r in range(rows) for c in range(cols)])
        np.testing.assert_allclose(got - pe, want, atol=1e-12)
        # stacked rows are the single-token definition
        one = O.embed_token(img, P, 1, 2, w[f"w_embed{lvl}"], w[f"b_embed{lvl}"])
        np.testing.assert_allclose(got[1 * cols + 2], one, atol=1e-13)


def test_embed_per_pixel_brute_force():
    rng = np.random.default_rng(0)
    img = rng.uniform(size=(3, 8, 8)).astype(np.float32)
    w = rng.standard_normal((4, 3 * 4 * 4)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    got = O.embed_token(img, 4, 1, 0, w, b)
    pe = O.pos_encoding(4, 1, 0, 8, 8, 4)
    for o in range(4):
        acc = float(b[o])
        for c in range(3):
            for r in range(4):
                for x in range(4):
                    acc += float(w[o, c * 16 + r * 4 + x]) * float(img[c, 4 + r, x])
        assert abs(acc + pe[o] - got[o]) < 1e-12


def test_coarse_cache_reuse_equals_recompute(tiny_cfg):
    cfg = tiny_cfg
    wl = _wl(cfg)
    tok, cu, _ = O.select_fine(wl["boxes"], wl["tier"], wl["box_offsets"],
                               cfg.B, cfg.H, cfg.W, cfg.patch)
    x0, _ = O.coarse_encode(wl["images"], cfg.patch, wl["weights"], cfg.heads)
    n0 = cfg.n_cells(0)
    for i in range(cfg.B):
        t = tok[cu[i]:cu[i + 1]]
        a = O.embed_frame(wl["images"][i], t, cfg.patch, wl["weights"], x0[i * n0:(i + 1) * n0])
        b = O.embed_frame(wl["images"][i], t, cfg.patch, wl["weights"], None)
        np.testing.assert_allclose(a, b, atol=1e-13)
        assert (t[:, 0] == 0).any() and (t[:, 0] == 1).any()


# ----------------------------------------------------------------- layer pieces
def test_layer_norm_and_gelu_against_library():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 24)) * 3 + 1
    g = rng.standard_normal(24).astype(np.float32)
    b = rng.standard_normal(24).astype(np.float32)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (24,),
                                          torch.from_numpy(g).double(),
                                          torch.from_numpy(b).double(), 1e-5).numpy()
    np.testing.assert_allclose(O.layer_norm(x, g, b), want, atol=1e-13)
    y = O.layer_norm(x, np.ones(24, np.float32), np.zeros(24, np.float32), eps=0.0)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose((y ** 2).mean(axis=1), 1, atol=1e-12)
    np.testing.assert_allclose(O.gelu(x), torch.nn.functional.gelu(torch.from_numpy(x)).numpy(),
                               atol=1e-14)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    assert abs(O.gelu(np.array([-1.0]))[0] + 0.15865525393145707) < 1e-15


def test_softmax_rows_sum_to_one():
    rng = np.random.default_rng(2)
    s = rng.standard_normal((9, 13)) * 30
    p = O.softmax_rows(s)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-14)
    assert (p >= 0).all()
    assert p[3].argmax() == s[3].argmax()


def _rand_attn(rng, T, d, scale=0.5):
    a = rng.standard_normal((T, d))
    w_qkv = (rng.standard_normal((3 * d, d)) * scale).astype(np.float32)
    b_qkv = (rng.standard_normal(3 * d) * scale).astype(np.float32)
    w_o = (rng.standard_normal((d, d)) * scale).astype(np.float32)
    b_o = (rng.standard_normal(d) * scale).astype(np.float32)
    return a, w_qkv, b_qkv, w_o, b_o


def test_attention_brute_force_loops():
    rng = np.random.default_rng(3)
    T, d, h = 5, 8, 2
    dh = d // h
    a, w_qkv, b_qkv, w_o, b_o = _rand_attn(rng, T, d)
    got = O.self_attention(a, w_qkv, b_qkv, w_o, b_o, h)
    qkv = [[sum(a[t, j] * float(w_qkv[o, j]) for j in range(d)) + float(b_qkv[o])
            for o in range(3 * d)] for t in range(T)]
    ctx = [[0.0] * d for _ in range(T)]
    for hh in range(h):
        for t in range(T):
            logits = [sum(qkv[t][hh * dh + i] * qkv[s][d + hh * dh + i] for i in range(dh))
                      / math.sqrt(dh) for s in range(T)]
            z = sum(math.exp(l) for l in logits)
            for i in range(dh):
                ctx[t][hh * dh + i] = sum(math.exp(logits[s]) / z * qkv[s][2 * d + hh * dh + i]
                                          for s in range(T))
    want = [[sum(ctx[t][j] * float(w_o[o, j]) for j in range(d)) + float(b_o[o])
             for o in range(d)] for t in range(T)]
    np.testing.assert_allclose(got, np.asarray(want), atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(4)
    T, d, h = 6, 8, 2
    a, w_qkv, b_qkv, w_o, b_o = _rand_attn(rng, T, d)
    # zero query projection -> uniform weights -> every row is the mean value vector
    wq0, bq0 = w_qkv.copy(), b_qkv.copy()
    wq0[:d], bq0[:d] = 0, 0
    v = a @ w_qkv[2 * d:].astype(np.float64).T + b_qkv[2 * d:]
    want = v.mean(axis=0) @ w_o.astype(np.float64).T + b_o
    got = O.self_attention(a, wq0, bq0, w_o, b_o, h)
    np.testing.assert_allclose(got, np.tile(want, (T, 1)), atol=1e-13)
    # a single token attends to itself only
    got1 = O.self_attention(a[:1], w_qkv, b_qkv, w_o, b_o, h)
    np.testing.assert_allclose(got1[0], v[0] @ w_o.astype(np.float64).T + b_o, atol=1e-13)
    # token order does not matter (permutation equivariance)
    perm = rng.permutation(T)
    full = O.self_attention(a, w_qkv, b_qkv, w_o, b_o, h)
    np.testing.assert_allclose(O.self_attention(a[perm], w_qkv, b_qkv, w_o, b_o, h),
                               full[perm], atol=1e-13)


def test_attention_against_library_mha():
    rng = np.random.default_rng(5)
    T, d, h = 11, 16, 4
    a, w_qkv, b_qkv, w_o, b_o = _rand_attn(rng, T, d)
    mha = torch.nn.MultiheadAttention(d, h, batch_first=True, dtype=torch.float64)
    with torch.no_grad():
        mha.in_proj_weight.copy_(torch.from_numpy(w_qkv).double())
        mha.in_proj_bias.copy_(torch.from_numpy(b_qkv).double())
        mha.out_proj.weight.copy_(torch.from_numpy(w_o).double())
        mha.out_proj.bias.copy_(torch.from_numpy(b_o).double())
        ta = torch.from_numpy(a)[None]
        want, attn = mha(ta, ta, ta, need_weights=True)
    np.testing.assert_allclose(O.self_attention(a, w_qkv, b_qkv, w_o, b_o, h),
                               want[0].numpy(), atol=1e-12)
    np.testing.assert_allclose(attn[0].sum(dim=-1).numpy(), 1.0, atol=1e-12)


def _torch_encoder(cfg, w):
    layer = torch.nn.TransformerEncoderLayer(
        cfg.d, cfg.heads, cfg.ffn, dropout=0.0, activation="gelu", layer_norm_eps=1e-5,
        batch_first=True, norm_first=True, dtype=torch.float64)
    enc = torch.nn.TransformerEncoder(layer, cfg.layers,
                                      norm=torch.nn.LayerNorm(cfg.d, eps=1e-5, dtype=torch.float64),
                                      enable_nested_tensor=False)
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    with torch.no_grad():
        for l, lay in enumerate(enc.layers):
            lay.self_attn.in_proj_weight.copy_(t(w["w_qkv"][l]))
            lay.self_attn.in_proj_bias.copy_(t(w["b_qkv"][l]))
            lay.self_attn.out_proj.weight.copy_(t(w["w_o"][l]))
            lay.self_attn.out_proj.bias.copy_(t(w["b_o"][l]))
            lay.linear1.weight.copy_(t(w["w_ff1"][l])); lay.linear1.bias.copy_(t(w["b_ff1"][l]))
            lay.linear2.weight.copy_(t(w["w_ff2"][l])); lay.linear2.bias.copy_(t(w["b_ff2"][l]))
            lay.norm1.weight.copy_(t(w["ln1_g"][l])); lay.norm1.bias.copy_(t(w["ln1_b"][l]))
            lay.norm2.weight.copy_(t(w["ln2_g"][l])); lay.norm2.bias.copy_(t(w["ln2_b"][l]))
        enc.norm.weight.copy_(t(w["lnf_g"])); enc.norm.bias.copy_(t(w["lnf_b"]))
    return enc.train(False)


@pytest.mark.parametrize("sharp", [False, True])
def test_encoder_against_library_pre_ln_stack(tiny_cfg, sharp):
    cfg = tiny_cfg
    w = synth.make_weights(cfg, 21, sharp=sharp, std=0.3)
    rng = np.random.default_rng(6)
    x = rng.standard_normal((19, cfg.d))
    enc = _torch_encoder(cfg, w)
    with torch.no_grad():
        want = enc(torch.from_numpy(x)[None])[0].numpy()
    np.testing.assert_allclose(O.encode_sequence(x, w, cfg.heads), want, atol=1e-11)


# ----------------------------------------------------------------- invariants of A1-A3
def test_no_roi_gives_coarse_encoder(tiny_cfg):
    cfg = tiny_cfg
    wl = _wl(cfg)
    none = np.zeros((0, 4), np.int32), np.zeros(0, np.uint8), np.zeros(cfg.B + 1, np.int32)
    yc, ym, tok, cu, counts = O.multilevel_batch(wl["images"], *none, cfg.patch,
                                                 wl["weights"], cfg.heads)
    assert cu.tolist() == [i * cfg.n_cells(0) for i in range(cfg.B + 1)]
    np.testing.assert_array_equal(ym, yc)


def test_all_critical_gives_plain_fine_vit(tiny_cfg):
    cfg = tiny_cfg
    wl = _wl(cfg)
    w = wl["weights"]
    boxes = np.tile(np.asarray([[0, 0, cfg.W, cfg.H]], np.int32), (cfg.B, 1))
    tier = np.full(cfg.B, cfg.n_levels - 1, np.uint8)
    offs = np.arange(cfg.B + 1, dtype=np.int32)
    _, ym, tok, cu, _ = O.multilevel_batch(wl["images"], boxes, tier, offs, cfg.patch,
                                           w, cfg.heads)
    top = cfg.n_levels - 1
    P = cfg.patch[top]
    rows, cols = cfg.grid(top)
    assert cu.tolist() == [i * rows * cols for i in range(cfg.B + 1)]
    enc = _torch_encoder(cfg, w)
    pe = np.stack([O.pos_encoding(P, r, c, cfg.H, cfg.W, cfg.d)
                   for r in range(rows) for c in range(cols)])
    with torch.no_grad():
        feat = torch.nn.functional.conv2d(
            torch.from_numpy(wl["images"]).double(),
            torch.from_numpy(w[f"w_embed{top}"]).double().reshape(cfg.d, 3, P, P),
            torch.from_numpy(w[f"b_embed{top}"]).double(), stride=P)       # [B,d,rows,cols]
        x = feat.flatten(2).transpose(1, 2) + torch.from_numpy(pe)[None]
        want = enc(x).reshape(cfg.B * rows * cols, cfg.d).numpy()
    np.testing.assert_allclose(ym, want, atol=1e-11)


def test_batched_equals_frame_by_frame_and_ignores_neighbours(tiny_cfg):
    cfg = tiny_cfg
    wl = _wl(cfg, sharp=True)
    w = wl["weights"]
    yc, ym, tok, cu, _ = O.multilevel_batch(wl["images"], wl["boxes"], wl["tier"],
                                            wl["box_offsets"], cfg.patch, w, cfg.heads)
    assert len(set(np.diff(cu).tolist())) > 1, "frames should have different lengths"
    for i in range(cfg.B):
        lo, hi = wl["box_offsets"][i], wl["box_offsets"][i + 1]
        one = O.multilevel_batch(wl["images"][i:i + 1], wl["boxes"][lo:hi], wl["tier"][lo:hi],
                                 np.asarray([0, hi - lo], np.int32), cfg.patch, w, cfg.heads)
        np.testing.assert_array_equal(one[1], ym[cu[i]:cu[i + 1]])
    # replacing frame 1 leaves frame 0's result untouched
    other = wl["images"].copy()
    other[1] = 1.0 - other[1]
    ym2 = O.multilevel_batch(other, wl["boxes"], wl["tier"], wl["box_offsets"], cfg.patch,
                             w, cfg.heads)[1]
    np.testing.assert_array_equal(ym2[:cu[1]], ym[:cu[1]])
    assert np.abs(ym2[cu[1]:] - ym[cu[1]:]).max() > 1e-3


def test_padded_masked_batch_equals_variable_length(tiny_cfg):
    cfg = tiny_cfg
    wl = _wl(cfg, sharp=True)
    w = wl["weights"]
    tok, cu, _ = O.select_fine(wl["boxes"], wl["tier"], wl["box_offsets"],
                               cfg.B, cfg.H, cfg.W, cfg.patch)
    xs = [O.embed_frame(wl["images"][i], tok[cu[i]:cu[i + 1]], cfg.patch, w)
          for i in range(cfg.B)]
    padded = O.encode_padded(xs, w, cfg.heads)
    for x, y in zip(xs, padded):
        np.testing.assert_allclose(y, O.encode_sequence(x, w, cfg.heads), atol=1e-12)


def test_encoder_is_permutation_equivariant(tiny_cfg):
    cfg = tiny_cfg
    w = synth.make_weights(cfg, 5, sharp=True)
    rng = np.random.default_rng(8)
    x = rng.standard_normal((23, cfg.d))
    perm = rng.permutation(23)
    np.testing.assert_allclose(O.encode_sequence(x[perm], w, cfg.heads),
                               O.encode_sequence(x, w, cfg.heads)[perm], atol=1e-12)


def test_sharp_weights_give_peaked_attention(tiny_cfg):
    # the test-only weight set must actually move the softmax away from uniform
    cfg = synth.replace(tiny_cfg, d=64, heads=2)
    w = synth.make_weights(cfg, 9, sharp=True)
    rng = np.random.default_rng(9)
    a = rng.standard_normal((50, cfg.d))
    qkv = a @ w["w_qkv"][0].astype(np.float64).T
    s = qkv[:, :32] @ qkv[:, 64:96].T / math.sqrt(32)
    assert 1.5 < s.std() < 6.0
