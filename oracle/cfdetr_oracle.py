"""CPU oracle for the coarse-to-fine detection-transformer encoder (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP library is compared against.  Only the test-suite, the smoke check and the
benchmark's CPU-baseline leg may import it; the product never does, and this
file imports nothing from the product.

What it computes, and where the paper states it:

* tokens are patch embeddings: the image is cut into a grid of patches and each
  patch becomes one vector (Sec. II-A, first paragraph on DETR);
* the encoder is self-attention in which every token of a frame attends to
  every other token of the same frame (Sec. II-A);
* the coarse pass (A1, Sec. III-B) runs the encoder on the coarse grid of every
  frame of an image-level batch;
* the selective fine pass (A2, Sec. III-B) re-partitions only the regions of
  interest into finer patches and keeps the coarse-stage tokens everywhere
  else, so each frame gets a mixed-granularity token set;
* multi-level batching (A3, Sec. III-B) runs several frames' token sets, of
  different lengths, through the encoder together; batching is a latency
  device and must not change any frame's result;
* learned object queries attend to the encoded tokens in a decoder and come out as
  candidate boxes with a confidence (Sec. II-A);
* the coarse stage's object queries decide whether a frame is easy or hard
  (A1: average confidence of the queries that are not already certain) and,
  for hard frames, propose the regions to refine (A2: the boxes of the
  queries of intermediate confidence).

The paper fixes the structure only.  Every numerical choice below that it is
silent on (linear patch projection, quadtree split rule, level-major token
order, centre-based 2-D sinusoidal positions, pre-LN layers with exact GELU)
is a stated reading; each reading is listed with its reason in the design
notes of this repository and is pinned by closed forms, invariants, brute
force or a library special case in tests/test_oracle_*.py.  Nothing in this
file is marked "parity unpinned".

All arithmetic is float64.  Library primitives used as steps: matrix product
(numpy ``@``), ``numpy.exp``, ``scipy.special.erf``.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf

LN_EPS = 1e-5


# --------------------------------------------------------------------------
# A2: which cells are refined, and in what order the tokens come out
# --------------------------------------------------------------------------
def _clip_boxes(boxes: np.ndarray, tier: np.ndarray, H: int, W: int):
    """Clip half-open pixel rectangles to the frame; drop the empty ones."""
    b = np.asarray(boxes, dtype=np.int64).reshape(-1, 4)
    t = np.asarray(tier, dtype=np.int64).reshape(-1)
    x0, y0 = np.maximum(b[:, 0], 0), np.maximum(b[:, 1], 0)
    x1, y1 = np.minimum(b[:, 2], W), np.minimum(b[:, 3], H)
    keep = (x1 > x0) & (y1 > y0)
    return x0[keep], y0[keep], x1[keep], y1[keep], t[keep]


def _cell_hits(clipped, level: int, P: int, row: int, col: int) -> bool:
    """Does any box asking for a level finer than ``level`` overlap this cell?

    A box that is empty after clipping to the frame overlaps nothing (A2: only
    the query-defined regions are re-partitioned).
    """
    x0, y0, x1, y1, t = clipped
    hit = ((t > level) & (x0 < (col + 1) * P) & (x1 > col * P)
           & (y0 < (row + 1) * P) & (y1 > row * P))
    return bool(hit.any())


def select_frame(boxes: np.ndarray, tier: np.ndarray, H: int, W: int,
                 patch: Sequence[int]) -> List[Tuple[int, int, int]]:
    """Leaf cells of one frame as (level, row, col), level-major then row-major.

    A2 (Sec. III-B): regions of interest are re-partitioned into finer
    patches, everything else keeps its coarse token.  Reading for boxes that
    cut through cells and for more than two granularities: a cell at a
    non-finest level is replaced by its four children iff a box of this frame
    whose tier is finer than the cell's level overlaps it; children are tested
    the same way.  The leaves tile the frame exactly.
    """
    n = len(patch)
    leaves: List[Tuple[int, int, int]] = []
    clipped = _clip_boxes(boxes, tier, H, W)

    def visit(level: int, row: int, col: int) -> None:
        if level < n - 1 and _cell_hits(clipped, level, patch[level], row, col):
            for dr in (0, 1):
                for dc in (0, 1):
                    visit(level + 1, 2 * row + dr, 2 * col + dc)
        else:
            leaves.append((level, row, col))

    for r in range(H // patch[0]):
        for c in range(W // patch[0]):
            visit(0, r, c)
    leaves.sort()            # (level, row, col): coarse first, row-major inside a level
    return leaves


def select_fine(boxes: np.ndarray, tier: np.ndarray, box_offsets: np.ndarray,
                B: int, H: int, W: int, patch: Sequence[int],
                hard: Optional[np.ndarray] = None):
    """A2 over a batch: token table, per-frame offsets, per-level counts.

    Returns (tok int64 [T,3] rows (level,row,col), cu_seqlens int64 [B+1],
    level_counts int64 [B, n_levels]).  Frames are concatenated in batch order.

    ``hard`` (optional, one flag per frame) is the outcome of the difficulty test of
    A1 (Sec. III-B): an easy frame is finished after the coarse stage, its fine-grained
    processing is skipped, so it contributes no token at all.
    """
    n = len(patch)
    toks: List[Tuple[int, int, int]] = []
    cu = [0]
    counts = np.zeros((B, n), dtype=np.int64)
    for i in range(B):
        if hard is not None and not hard[i]:
            cu.append(len(toks))
            continue
        lo, hi = int(box_offsets[i]), int(box_offsets[i + 1])
        leaves = select_frame(boxes[lo:hi], tier[lo:hi], H, W, patch)
        for (lvl, _, _) in leaves:
            counts[i, lvl] += 1
        toks.extend(leaves)
        cu.append(len(toks))
    return (np.asarray(toks, dtype=np.int64).reshape(-1, 3),
            np.asarray(cu, dtype=np.int64), counts)


# --------------------------------------------------------------------------
# A1 (difficulty of a frame) and A2 (regions of interest) from the coarse
# stage's object queries
# --------------------------------------------------------------------------
def frame_hardness(conf: np.ndarray, tau_hi: float, tau_lo: float) -> Tuple[bool, float]:
    """Difficulty of one frame from its query confidences (Sec. III-B, A1).

    Queries above ``tau_hi`` are the prominent, already certain objects and are
    left out; the confidences of all the others are averaged; a frame whose
    average is below ``tau_lo`` is easy, any other frame is hard.  Reading
    where the paper is silent: with no query left the average is 0 (easy).
    Returns (hard, average)."""
    c = np.asarray(conf, dtype=np.float64)
    rest = c[~(c > tau_hi)]
    mean = float(rest.sum() / len(rest)) if len(rest) else 0.0
    return (not mean < tau_lo), mean


def roi_box(cx: float, cy: float, w: float, h: float, H: int, W: int,
            scale: float = 1.0, min_side: float = 0.0) -> Tuple[int, int, int, int]:
    """Pixel rectangle of one query box (Sec. III-B, A2: regions are proposed from
    the location and size of the queries).

    Readings: (cx, cy, w, h) are the centre and the size as fractions of the frame;
    the region is the box scaled by ``scale`` about its centre and at least
    ``min_side`` pixels wide and high (the adjustable region size of the paper's
    draft); the half-open pixel rectangle is the smallest one that covers it
    (lower edges rounded down, upper edges up), clipped to the frame.  The
    arithmetic is float64 in this order: half = max(0.5*scale*size*extent,
    0.5*min_side); edges = centre*extent -/+ half."""
    half_w = max(0.5 * scale * w * W, 0.5 * min_side)
    half_h = max(0.5 * scale * h * H, 0.5 * min_side)
    x0 = math.floor(cx * W - half_w)
    x1 = math.ceil(cx * W + half_w)
    y0 = math.floor(cy * H - half_h)
    y1 = math.ceil(cy * H + half_h)
    return (min(max(x0, 0), W), min(max(y0, 0), H), min(max(x1, 0), W), min(max(y1, 0), H))


def propose_rois(queries: np.ndarray, H: int, W: int, tau_hi: float, tau_lo: float,
                 tier: int, scale: float = 1.0, min_side: float = 0.0):
    """A1 difficulty test and A2 region proposal for a batch (Sec. III-B).

    queries [B, Q, 5] = (cx, cy, w, h, c).  An easy frame proposes nothing (its
    fine pass is skipped or equals its coarse pass); a hard frame proposes one
    region per query of intermediate confidence, tau_lo < c <= tau_hi, in query
    order, all with the refinement level ``tier``.
    Returns boxes int32 [n,4], tier uint8 [n], box_offsets int32 [B+1],
    hard int32 [B], mean float64 [B]."""
    q = np.asarray(queries, dtype=np.float64)
    B = q.shape[0]
    boxes: List[Tuple[int, int, int, int]] = []
    offs = [0]
    hard = np.zeros(B, dtype=np.int32)
    mean = np.zeros(B, dtype=np.float64)
    for f in range(B):
        is_hard, mean[f] = frame_hardness(q[f, :, 4], tau_hi, tau_lo)
        hard[f] = int(is_hard)
        if is_hard:
            for k in range(q.shape[1]):
                cx, cy, w, h, c = q[f, k]
                if tau_lo < c <= tau_hi:
                    boxes.append(roi_box(cx, cy, w, h, H, W, scale, min_side))
        offs.append(len(boxes))
    b = np.asarray(boxes, dtype=np.int32).reshape(-1, 4)
    return (b, np.full(len(b), tier, dtype=np.uint8), np.asarray(offs, dtype=np.int32), hard, mean)


def merge_detections(coarse: np.ndarray, fine: np.ndarray, hard: np.ndarray, tau_hi: float,
                     tau_fine: float):
    """Final detections of a batch (Sec. III-B, last step of A2: confident coarse
    detections are kept, the fine stage's detections replace the uncertain ones).

    coarse, fine [B, Q, 5] = (cx, cy, w, h, c) from the coarse and the fine stage; hard [B]
    from the difficulty test.  Frame f keeps its coarse queries with c > tau_hi, in query
    order; a hard frame then adds its fine-stage queries with c > tau_fine, in query
    order (an easy frame has no fine stage: its ``fine`` rows are ignored).
    Returns det float32 [B, 2Q, 5] (rows past the count are zero), src uint8 [B, 2Q]
    (0 = coarse stage, 1 = fine stage, 255 past the count), count int32 [B]."""
    c32 = np.asarray(coarse, dtype=np.float32)
    f32 = np.asarray(fine, dtype=np.float32)
    B, Q = c32.shape[:2]
    det = np.zeros((B, 2 * Q, 5), dtype=np.float32)
    src = np.full((B, 2 * Q), 255, dtype=np.uint8)
    count = np.zeros(B, dtype=np.int32)
    for f in range(B):
        n = 0
        for k in range(Q):
            if float(c32[f, k, 4]) > tau_hi:
                det[f, n] = c32[f, k]
                src[f, n] = 0
                n += 1
        if hard[f]:
            for k in range(Q):
                if float(f32[f, k, 4]) > tau_fine:
                    det[f, n] = f32[f, k]
                    src[f, n] = 1
                    n += 1
        count[f] = n
    return det, src, count


def pack_tok_desc(tok: np.ndarray) -> np.ndarray:
    """(level,row,col) -> one int32 per token: level<<28 | row<<14 | col."""
    t = np.asarray(tok, dtype=np.int64)
    return ((t[:, 0] << 28) | (t[:, 1] << 14) | t[:, 2]).astype(np.int32)


# --------------------------------------------------------------------------
# tokens: patch embedding + position
# --------------------------------------------------------------------------
def pos_encoding(P: int, row: int, col: int, H: int, W: int, d: int) -> np.ndarray:
    """2-D sinusoidal position of a cell, taken at the cell's centre.

    One coordinate system serves every granularity: u, v in (0,1) are the
    centre of the cell in normalised frame coordinates.  The first half of the
    vector encodes v (vertical), the second half u (horizontal), each as
    interleaved (sin, cos) pairs at frequencies 10000^(-2j/D), D = d/2.
    """
    D = d // 2
    v = (row + 0.5) * P / H
    u = (col + 0.5) * P / W
    pe = np.empty(d, dtype=np.float64)
    for j in range(D // 2):
        omega = 10000.0 ** (-2.0 * j / D)
        pe[2 * j] = math.sin(2.0 * math.pi * v * omega)
        pe[2 * j + 1] = math.cos(2.0 * math.pi * v * omega)
        pe[D + 2 * j] = math.sin(2.0 * math.pi * u * omega)
        pe[D + 2 * j + 1] = math.cos(2.0 * math.pi * u * omega)
    return pe


def embed_token(image: np.ndarray, P: int, row: int, col: int,
                w: np.ndarray, b: np.ndarray) -> np.ndarray:
    """One token: linear projection of the flattened patch, plus bias, plus position.

    Sec. II-A: each patch is turned from RGB into one vector.  Reading: the
    frame is planar [3,H,W]; the patch is flattened (channel, row, column) and
    projected by that granularity's own matrix w [d, 3*P*P].
    """
    _, H, W = image.shape
    pix = image[:, row * P:(row + 1) * P, col * P:(col + 1) * P].astype(np.float64)
    return (w.astype(np.float64) @ pix.reshape(-1) + b.astype(np.float64)
            + pos_encoding(P, row, col, H, W, w.shape[0]))


def embed_frame(image: np.ndarray, tok: np.ndarray, patch: Sequence[int],
                weights: Dict[str, np.ndarray],
                x0_frame: Optional[np.ndarray] = None) -> np.ndarray:
    """Token matrix [T_i, d] of one frame for a given leaf table.

    A2/A3: tokens of unrefined areas are the coarse-stage tokens, reused (what
    is cached is the embedding that enters the encoder, so that no feature
    extraction is repeated); refined areas get new tokens at their own
    granularity.  ``x0_frame`` [N0, d] is that cache; without it coarse leaves
    are embedded again, which must give the same numbers.

    Same arithmetic as ``embed_token`` for every row; the rows of one
    granularity are stacked so that their projection is one matrix product.
    """
    _, H, W = image.shape
    d = weights["b_embed0"].shape[0]
    cols0 = W // patch[0]
    tok = np.asarray(tok, dtype=np.int64).reshape(-1, 3)
    x = np.empty((len(tok), d), dtype=np.float64)
    for lvl, P in enumerate(patch):
        idx = np.nonzero(tok[:, 0] == lvl)[0]
        if len(idx) == 0:
            continue
        if lvl == 0 and x0_frame is not None:
            x[idx] = x0_frame[tok[idx, 1] * cols0 + tok[idx, 2]]
            continue
        pix = np.empty((len(idx), 3 * P * P), dtype=np.float64)
        pe = np.empty((len(idx), d), dtype=np.float64)
        for n, t in enumerate(idx):
            row, col = int(tok[t, 1]), int(tok[t, 2])
            pix[n] = image[:, row * P:(row + 1) * P, col * P:(col + 1) * P].reshape(-1)
            pe[n] = pos_encoding(P, row, col, H, W, d)
        x[idx] = (pix @ weights[f"w_embed{lvl}"].astype(np.float64).T
                  + weights[f"b_embed{lvl}"].astype(np.float64) + pe)
    return x


# --------------------------------------------------------------------------
# encoder
# --------------------------------------------------------------------------
def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float = LN_EPS) -> np.ndarray:
    """Per-row normalisation with biased variance, then gain and shift."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g.astype(np.float64) + b.astype(np.float64)


def gelu(x: np.ndarray) -> np.ndarray:
    """Exact GELU: x * Phi(x)."""
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def self_attention(a: np.ndarray, w_qkv: np.ndarray, b_qkv: np.ndarray,
                   w_o: np.ndarray, b_o: np.ndarray, heads: int,
                   key_mask: Optional[np.ndarray] = None) -> np.ndarray:
    """Multi-head self-attention of one sequence a [T, d] (Sec. II-A).

    w_qkv [3d, d] stacks the query, key and value projections; head h owns
    columns h*dh .. (h+1)*dh of each.  The T x T score matrix is materialised.
    ``key_mask`` (bool [T], True = real token) removes padded keys.
    """
    T, d = a.shape
    dh = d // heads
    qkv = a @ w_qkv.astype(np.float64).T + b_qkv.astype(np.float64)
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    out = np.empty((T, d), dtype=np.float64)
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = q[:, sl] @ k[:, sl].T / math.sqrt(dh)
        if key_mask is not None:
            s = np.where(key_mask[None, :], s, -np.inf)
        out[:, sl] = softmax_rows(s) @ v[:, sl]
    return out @ w_o.astype(np.float64).T + b_o.astype(np.float64)


def encoder_layer(x: np.ndarray, weights: Dict[str, np.ndarray], l: int, heads: int,
                  key_mask: Optional[np.ndarray] = None) -> np.ndarray:
    """One pre-LN layer: x + MHA(LN1 x), then x + W2 GELU(W1 LN2 x)."""
    w = weights
    a = layer_norm(x, w["ln1_g"][l], w["ln1_b"][l])
    x = x + self_attention(a, w["w_qkv"][l], w["b_qkv"][l], w["w_o"][l], w["b_o"][l],
                           heads, key_mask)
    m = layer_norm(x, w["ln2_g"][l], w["ln2_b"][l])
    hdn = gelu(m @ w["w_ff1"][l].astype(np.float64).T + w["b_ff1"][l].astype(np.float64))
    return x + hdn @ w["w_ff2"][l].astype(np.float64).T + w["b_ff2"][l].astype(np.float64)


def encode_sequence(x: np.ndarray, weights: Dict[str, np.ndarray], heads: int,
                    key_mask: Optional[np.ndarray] = None) -> np.ndarray:
    """All layers plus the final LayerNorm over one frame's tokens."""
    for l in range(weights["w_qkv"].shape[0]):
        x = encoder_layer(x, weights, l, heads, key_mask)
    return layer_norm(x, weights["lnf_g"], weights["lnf_b"])


# --------------------------------------------------------------------------
# decoder: learned object queries read the encoded tokens of their frame and
# become candidate boxes with a confidence (Sec. II-A)
# --------------------------------------------------------------------------
def cross_attention(a: np.ndarray, mem: np.ndarray, w_q: np.ndarray, b_q: np.ndarray,
                    w_kv: np.ndarray, b_kv: np.ndarray, w_o: np.ndarray, b_o: np.ndarray,
                    heads: int) -> np.ndarray:
    """Multi-head attention of queries a [Q, d] over the tokens mem [T, d] of the same
    frame (Sec. II-A: object queries attend to the encoded patches).  w_kv [2d, d] stacks
    the key and value projections."""
    Q, d = a.shape
    dh = d // heads
    q = a @ w_q.astype(np.float64).T + b_q.astype(np.float64)
    kv = mem @ w_kv.astype(np.float64).T + b_kv.astype(np.float64)
    k, v = kv[:, :d], kv[:, d:]
    out = np.empty((Q, d), dtype=np.float64)
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        out[:, sl] = softmax_rows(q[:, sl] @ k[:, sl].T / math.sqrt(dh)) @ v[:, sl]
    return out @ w_o.astype(np.float64).T + b_o.astype(np.float64)


def decode_frame(mem: np.ndarray, dw: Dict[str, np.ndarray], heads: int) -> np.ndarray:
    """Object queries of one frame from its encoded tokens mem [T, d]; returns [Q, 5] =
    (cx, cy, w, h, c), all in (0, 1).

    Readings (the paper describes the DETR pipeline, Sec. II-A, and fixes no layer
    details): the queries start as learned vectors; every layer is pre-LN,
    x += SelfAttn(LN1 x); x += CrossAttn(LN2 x, mem); x += W2 GELU(W1 LN3 x); a final
    LayerNorm; no positional term beyond what the tokens already carry.  Heads: the
    confidence is the sigmoid of one linear output, the box the sigmoid of a three-layer
    perceptron with ReLU (centre and size as fractions of the frame)."""
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    x = f64(dw["query_embed"]).copy()
    for l in range(dw["w_qkv"].shape[0]):
        a = layer_norm(x, dw["ln1_g"][l], dw["ln1_b"][l])
        x = x + self_attention(a, dw["w_qkv"][l], dw["b_qkv"][l], dw["w_o"][l], dw["b_o"][l], heads)
        a = layer_norm(x, dw["ln2_g"][l], dw["ln2_b"][l])
        x = x + cross_attention(a, mem, dw["w_q"][l], dw["b_q"][l], dw["w_kv"][l], dw["b_kv"][l],
                                dw["w_o2"][l], dw["b_o2"][l], heads)
        m = layer_norm(x, dw["ln3_g"][l], dw["ln3_b"][l])
        hdn = gelu(m @ f64(dw["w_ff1"][l]).T + f64(dw["b_ff1"][l]))
        x = x + hdn @ f64(dw["w_ff2"][l]).T + f64(dw["b_ff2"][l])
    z = layer_norm(x, dw["lnf_g"], dw["lnf_b"])
    sig = lambda u: 1.0 / (1.0 + np.exp(-u))
    conf = sig(z @ f64(dw["w_cls"]).T + f64(dw["b_cls"]))                      # [Q, 1]
    h1 = np.maximum(z @ f64(dw["w_box1"]).T + f64(dw["b_box1"]), 0.0)
    h2 = np.maximum(h1 @ f64(dw["w_box2"]).T + f64(dw["b_box2"]), 0.0)
    box = sig(h2 @ f64(dw["w_box3"]).T + f64(dw["b_box3"]))                    # [Q, 4]
    return np.concatenate([box, conf], axis=1)


def decode(memory: np.ndarray, cu_seqlens: np.ndarray, dw: Dict[str, np.ndarray],
           heads: int) -> np.ndarray:
    """decode_frame for every frame of a batch: memory [T, d] with frame i at rows
    cu_seqlens[i]..cu_seqlens[i+1]; returns [B, Q, 5].  Frames do not interact."""
    return np.stack([decode_frame(memory[cu_seqlens[f]:cu_seqlens[f + 1]], dw, heads)
                     for f in range(len(cu_seqlens) - 1)])


# --------------------------------------------------------------------------
# the four calls of the boundary, frame by frame
# --------------------------------------------------------------------------
def coarse_encode(images: np.ndarray, patch: Sequence[int],
                  weights: Dict[str, np.ndarray], heads: int):
    """A1: every frame on its coarse grid.  Returns (x0 [B*N0,d], y_coarse [B*N0,d])."""
    B, _, H, W = images.shape
    rows, cols = H // patch[0], W // patch[0]
    tok = np.asarray([(0, r, c) for r in range(rows) for c in range(cols)], dtype=np.int64)
    x0, y = [], []
    for i in range(B):
        xi = embed_frame(images[i], tok, patch, weights)
        x0.append(xi)
        y.append(encode_sequence(xi, weights, heads))
    return np.concatenate(x0), np.concatenate(y)


def fine_encode(images: np.ndarray, tok: np.ndarray, cu_seqlens: np.ndarray,
                patch: Sequence[int], weights: Dict[str, np.ndarray], heads: int,
                x0_cache: Optional[np.ndarray] = None) -> np.ndarray:
    """A2+A3: every frame on its own mixed-granularity token set.

    Frames are processed one at a time: a token only ever attends inside its
    own frame, so this is what any batched execution must reproduce.
    """
    B, _, H, W = images.shape
    n0 = (H // patch[0]) * (W // patch[0])
    ys = []
    for i in range(B):
        lo, hi = int(cu_seqlens[i]), int(cu_seqlens[i + 1])
        if hi == lo:
            continue
        x0f = None if x0_cache is None else x0_cache[i * n0:(i + 1) * n0]
        xi = embed_frame(images[i], tok[lo:hi], patch, weights, x0f)
        ys.append(encode_sequence(xi, weights, heads))
    d = weights["b_embed0"].shape[0]
    return np.concatenate(ys) if ys else np.zeros((0, d))


def multilevel_batch(images: np.ndarray, boxes: np.ndarray, tier: np.ndarray,
                     box_offsets: np.ndarray, patch: Sequence[int],
                     weights: Dict[str, np.ndarray], heads: int):
    """A1 -> A2 -> A3.  Returns (y_coarse, y_mixed, tok, cu_seqlens, level_counts)."""
    B, _, H, W = images.shape
    x0, y_coarse = coarse_encode(images, patch, weights, heads)
    tok, cu, counts = select_fine(boxes, tier, box_offsets, B, H, W, patch)
    y_mixed = fine_encode(images, tok, cu, patch, weights, heads, x0_cache=x0)
    return y_coarse, y_mixed, tok, cu, counts


def encode_padded(xs: List[np.ndarray], weights: Dict[str, np.ndarray], heads: int):
    """The paper's literal A3 batching: pad every frame's tokens with zero rows
    to the longest frame, run the batch, drop the padding.  Padded keys are
    masked out of the softmax (reading: batching changes latency, not results).
    """
    tmax = max(len(x) for x in xs)
    outs = []
    for x in xs:
        pad = np.zeros((tmax - len(x), x.shape[1]))
        mask = np.arange(tmax) < len(x)
        y = encode_sequence(np.concatenate([x, pad]), weights, heads, key_mask=mask)
        outs.append(y[: len(x)])
    return outs
