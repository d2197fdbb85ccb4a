"""Pins for the oracle's decoder (Sec. II-A: object queries attend to the encoded
patches and give boxes with a confidence): PyTorch's own pre-LN transformer decoder in
fp64 with the same weights, a pure-Python cross-attention, and invariants."""
import math

import numpy as np
import pytest
import torch

from oracle import cfdetr_oracle as O
from paper_2505_23317_amd import synth


def _cfg():
    return synth.Config("dec", 2, 64, 64, (16, 8), 32, 4, 1, 64, "f32", box_rule="single48")


def test_cross_attention_against_loops():
    rng = np.random.default_rng(0)
    d, heads, Q, T = 8, 2, 3, 5
    a, mem = rng.normal(size=(Q, d)), rng.normal(size=(T, d))
    wq, bq = rng.normal(size=(d, d)), rng.normal(size=d)
    wkv, bkv = rng.normal(size=(2 * d, d)), rng.normal(size=2 * d)
    wo, bo = rng.normal(size=(d, d)), rng.normal(size=d)
    got = O.cross_attention(a, mem, wq, bq, wkv, bkv, wo, bo, heads)
    dh = d // heads
    want = np.zeros((Q, d))
    for i in range(Q):
        ctx = np.zeros(d)
        for h in range(heads):
            q = [sum(a[i, c] * wq[h * dh + e, c] for c in range(d)) + bq[h * dh + e] for e in range(dh)]
            logits = []
            vals = []
            for t in range(T):
                k = [sum(mem[t, c] * wkv[h * dh + e, c] for c in range(d)) + bkv[h * dh + e] for e in range(dh)]
                v = [sum(mem[t, c] * wkv[d + h * dh + e, c] for c in range(d)) + bkv[d + h * dh + e] for e in range(dh)]
                logits.append(sum(q[e] * k[e] for e in range(dh)) / math.sqrt(dh))
                vals.append(v)
            mx = max(logits)
            p = [math.exp(l - mx) for l in logits]
            z = sum(p)
            for e in range(dh):
                ctx[h * dh + e] = sum(p[t] / z * vals[t][e] for t in range(T))
        want[i] = wo @ ctx + bo
    assert np.abs(got - want).max() < 1e-12


def test_decoder_against_torch():
    cfg = _cfg()
    dw = synth.make_decoder_weights(cfg, 1, n_queries=7, layers=2, std=0.3)
    d, heads, L = cfg.d, cfg.heads, 2
    rng = np.random.default_rng(3)
    mem = rng.normal(size=(11, d))
    layer = torch.nn.TransformerDecoderLayer(d, heads, cfg.ffn, dropout=0.0, activation="gelu",
                                             batch_first=True, norm_first=True, dtype=torch.float64)
    dec = torch.nn.TransformerDecoder(layer, L, norm=torch.nn.LayerNorm(d, dtype=torch.float64))
    T = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        for l, ly in enumerate(dec.layers):
            ly.self_attn.in_proj_weight.copy_(T(dw["w_qkv"][l]))
            ly.self_attn.in_proj_bias.copy_(T(dw["b_qkv"][l]))
            ly.self_attn.out_proj.weight.copy_(T(dw["w_o"][l]))
            ly.self_attn.out_proj.bias.copy_(T(dw["b_o"][l]))
            ly.multihead_attn.in_proj_weight.copy_(T(np.concatenate([dw["w_q"][l], dw["w_kv"][l]])))
            ly.multihead_attn.in_proj_bias.copy_(T(np.concatenate([dw["b_q"][l], dw["b_kv"][l]])))
            ly.multihead_attn.out_proj.weight.copy_(T(dw["w_o2"][l]))
            ly.multihead_attn.out_proj.bias.copy_(T(dw["b_o2"][l]))
            ly.linear1.weight.copy_(T(dw["w_ff1"][l])); ly.linear1.bias.copy_(T(dw["b_ff1"][l]))
            ly.linear2.weight.copy_(T(dw["w_ff2"][l])); ly.linear2.bias.copy_(T(dw["b_ff2"][l]))
            ly.norm1.weight.copy_(T(dw["ln1_g"][l])); ly.norm1.bias.copy_(T(dw["ln1_b"][l]))
            ly.norm2.weight.copy_(T(dw["ln2_g"][l])); ly.norm2.bias.copy_(T(dw["ln2_b"][l]))
            ly.norm3.weight.copy_(T(dw["ln3_g"][l])); ly.norm3.bias.copy_(T(dw["ln3_b"][l]))
        dec.norm.weight.copy_(T(dw["lnf_g"])); dec.norm.bias.copy_(T(dw["lnf_b"]))
        z = dec(T(dw["query_embed"])[None], T(mem)[None])[0]
        conf = torch.sigmoid(z @ T(dw["w_cls"]).T + T(dw["b_cls"]))
        h = torch.relu(z @ T(dw["w_box1"]).T + T(dw["b_box1"]))
        h = torch.relu(h @ T(dw["w_box2"]).T + T(dw["b_box2"]))
        box = torch.sigmoid(h @ T(dw["w_box3"]).T + T(dw["b_box3"]))
        want = torch.cat([box, conf], dim=1).numpy()
    got = O.decode_frame(mem, dw, heads)
    assert got.shape == (7, 5)
    assert np.abs(got - want).max() < 1e-12


def test_decoder_invariants():
    cfg = _cfg()
    dw = synth.make_decoder_weights(cfg, 2, n_queries=5, layers=1, std=0.3)
    rng = np.random.default_rng(4)
    mem = rng.normal(size=(9, cfg.d))
    out = O.decode_frame(mem, dw, cfg.heads)
    assert ((out > 0) & (out < 1)).all()
    # attention has no notion of token order: permuting the frame's tokens changes nothing
    perm = rng.permutation(9)
    assert np.abs(O.decode_frame(mem[perm], dw, cfg.heads) - out).max() < 1e-12
    # frames of a batch do not interact
    mem2 = rng.normal(size=(4, cfg.d))
    both = O.decode(np.concatenate([mem, mem2]), np.array([0, 9, 13]), dw, cfg.heads)
    assert np.abs(both[0] - out).max() == 0 and np.abs(both[1] - O.decode_frame(mem2, dw, cfg.heads)).max() == 0
    # with the value projection of the cross-attention zeroed, the tokens cannot matter
    dw0 = dict(dw)
    dw0["w_kv"] = dw["w_kv"].copy(); dw0["w_kv"][:, cfg.d:] = 0
    dw0["b_kv"] = dw["b_kv"].copy(); dw0["b_kv"][:, cfg.d:] = 0
    assert np.abs(O.decode_frame(mem, dw0, cfg.heads) - O.decode_frame(mem2, dw0, cfg.heads)).max() < 1e-12
    # a lower confidence bias lowers every confidence and no box
    dw1 = dict(dw); dw1["b_cls"] = dw["b_cls"] - 1.0
    low = O.decode_frame(mem, dw1, cfg.heads)
    assert (low[:, 4] < out[:, 4]).all() and np.array_equal(low[:, :4], out[:, :4])


def test_detection_heads_hand_worked():
    """The confidence and box heads against values worked by hand (closed-form sigmoids of
    logarithms; tests/golden/decoder_heads_worked_example.txt): no decoder layer, width 2, so
    the heads see the final LayerNorm of the query vectors.  A transposed matrix, a missing
    ReLU, a swapped output or a sign error in either head changes at least one value."""
    import os
    from fractions import Fraction
    want = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "decoder_heads_worked_example.txt")
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *vals = line.split()
            want[name] = [float(Fraction(v)) for v in vals]
    ln = math.log
    e = lambda *shape: np.zeros(shape)
    dw = {
        "query_embed": np.array([[1000.0, -1000.0], [-3000.0, 3000.0]]),
        "w_qkv": e(0, 6, 2),   # no layers: nothing else of a layer is read
        "lnf_g": np.array([1.0, 2.0]), "lnf_b": e(2),
        "w_cls": np.array([[ln(3), 0.0]]), "b_cls": e(1),
        "w_box1": np.array([[1.0, 1.0], [0.0, -1.0]]), "b_box1": np.array([2.0, -1.0]),
        "w_box2": np.array([[1.0, -1.0], [2.0, 0.0]]), "b_box2": np.array([0.0, -1.0]),
        "w_box3": np.array([[ln(3), 0.0], [0.0, ln(3)], [ln(2), -ln(2)], [0.0, 0.0]]),
        "b_box3": np.array([0.0, 0.0, 0.0, -ln(9)]),
    }
    got = O.decode_frame(np.ones((3, 2)), dw, 1)
    assert got.shape == (2, 5)
    assert np.abs(got[0] - want["A"]).max() < 1e-9
    assert np.abs(got[1] - want["B"]).max() < 1e-9
