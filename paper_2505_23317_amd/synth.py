"""Seeded synthetic workloads for the coarse-to-fine encoder.

This module only *draws inputs*: camera frames, RoI boxes with criticality
tiers, and random-init weights, shaped like the multi-camera AV workloads the
paper evaluates on (a handful of object boxes per frame, selective refinement
of a fraction of the frame; Sec. III-B, "Validating" paragraphs of A1/A2).  It
holds none of the method's arithmetic and imports neither the HIP binding nor
the CPU oracle; both consume the arrays it returns.

All matrices and images that a bf16 path will read are rounded to
bf16-representable values here, once, so that every consumer sees the same
numbers and only compute error is measured downstream.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

__all__ = [
    "Config", "CONFIGS", "config", "bf16_round", "bf16_bits", "make_weights",
    "make_frames", "make_workload", "make_queries", "make_decoder_weights", "replace",
]


@dataclass(frozen=True)
class Config:
    """Shape of one workload (one row of the benchmark configuration list)."""
    name: str
    B: int                      # cameras in the batch
    H: int
    W: int
    patch: Tuple[int, ...]      # coarse -> fine, each half the previous
    d: int                      # model width
    heads: int
    layers: int
    ffn: int
    image_dtype: str            # "f32" or "bf16"
    frac_lo: float = 0.0        # critical-area fraction range (None => Poisson boxes)
    frac_hi: float = 0.0
    box_rule: str = "poisson"   # "single48" | "poisson" | "fraction" | "tiered"
    box_lambda: float = 5.0
    side_lo: int = 32
    side_hi: int = 192

    @property
    def n_levels(self) -> int:
        return len(self.patch)

    def grid(self, level: int) -> Tuple[int, int]:
        p = self.patch[level]
        return self.H // p, self.W // p

    def n_cells(self, level: int) -> int:
        r, c = self.grid(level)
        return r * c

    @property
    def d_head(self) -> int:
        return self.d // self.heads


CONFIGS: Dict[int, Config] = {
    1: Config("cfg1_tiny", 1, 128, 128, (32, 16), 64, 2, 1, 128, "f32",
              box_rule="single48"),
    2: Config("cfg2_single_camera", 1, 640, 640, (32, 16), 256, 8, 6, 1024, "bf16",
              box_rule="poisson", box_lambda=5.0),
    3: Config("cfg3_six_cameras", 6, 640, 640, (32, 16), 256, 8, 6, 1024, "bf16",
              frac_lo=0.0, frac_hi=0.5, box_rule="fraction"),
    4: Config("cfg4_high_res", 4, 1280, 1280, (32, 16), 384, 6, 12, 1536, "bf16",
              frac_lo=0.0, frac_hi=1.0, box_rule="fraction"),
    5: Config("cfg5_three_level", 12, 1024, 1024, (64, 32, 16), 768, 12, 12, 3072, "bf16",
              box_rule="tiered", box_lambda=12.0, side_lo=64, side_hi=320),
}


def config(cfg_id: int) -> Config:
    return CONFIGS[cfg_id]


# --------------------------------------------------------------------------
# bf16 helpers (format conversion only)
# --------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16-representable float32."""
    bits = bf16_bits(x).astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).reshape(np.shape(x))


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def make_weights(cfg: Config, seed: int, sharp: bool = False,
                 std: float = 0.02) -> Dict[str, np.ndarray]:
    """Random-init encoder weights, N(0, std^2); LayerNorm gain 1 + N(0, std^2).

    Matrices are bf16-representable float32; vectors stay float32.  With
    ``sharp`` the query and key projections are scaled up so that attention
    logits have a spread of a few units (a peaked softmax), which the plain
    init does not produce; this set is for tests only.
    """
    rng = np.random.default_rng(seed)
    d, F, L = cfg.d, cfg.ffn, cfg.layers

    def mat(*shape):
        return bf16_round((rng.standard_normal(shape) * std).astype(np.float32))

    def vec(*shape):
        return (rng.standard_normal(shape) * std).astype(np.float32)

    w: Dict[str, np.ndarray] = {}
    for lvl, p in enumerate(cfg.patch):
        w[f"w_embed{lvl}"] = mat(d, 3 * p * p)
        w[f"b_embed{lvl}"] = vec(d)
    w["ln1_g"] = (1.0 + vec(L, d)).astype(np.float32)
    w["ln1_b"] = vec(L, d)
    w["w_qkv"] = mat(L, 3 * d, d)
    w["b_qkv"] = vec(L, 3 * d)
    w["w_o"] = mat(L, d, d)
    w["b_o"] = vec(L, d)
    w["ln2_g"] = (1.0 + vec(L, d)).astype(np.float32)
    w["ln2_b"] = vec(L, d)
    w["w_ff1"] = mat(L, F, d)
    w["b_ff1"] = vec(L, F)
    w["w_ff2"] = mat(L, d, F)
    w["b_ff2"] = vec(L, d)
    w["lnf_g"] = (1.0 + vec(d)).astype(np.float32)
    w["lnf_b"] = vec(d)
    if sharp:
        # LN output has unit variance per feature, so a q/k row with entries of
        # std s gives |q|,|k| components of std s*sqrt(d); logits q.k/sqrt(dh)
        # then have std ~ s^2 * d * sqrt(dh) / sqrt(dh).  Pick s for std ~ 3.
        s = float(np.sqrt(3.0 / d))
        qk = rng.standard_normal((L, 2 * d, d)).astype(np.float32) * s
        w["w_qkv"][:, : 2 * d, :] = bf16_round(qk)
    return w


# --------------------------------------------------------------------------
# frames and boxes
# --------------------------------------------------------------------------
def _rand_box(rng, H, W, lo, hi):
    bw = int(rng.integers(lo, hi + 1))
    bh = int(rng.integers(lo, hi + 1))
    bw, bh = min(bw, W), min(bh, H)
    x0 = int(rng.integers(0, W - bw + 1))
    y0 = int(rng.integers(0, H - bh + 1))
    return x0, y0, x0 + bw, y0 + bh


def _paint_frame(rng, cfg: Config, rects) -> np.ndarray:
    """Gaussian-noise background with constant-colour rectangles painted on."""
    img = rng.normal(0.5, 0.25, size=(3, cfg.H, cfg.W)).astype(np.float32)
    np.clip(img, 0.0, 1.0, out=img)
    for (x0, y0, x1, y1) in rects:
        colour = rng.uniform(0.0, 1.0, size=3).astype(np.float32)
        img[:, y0:y1, x0:x1] = colour[:, None, None]
    return img


def make_frames(cfg: Config, seed: int):
    """Draw B frames plus their RoI boxes and criticality tiers.

    Returns (images float32 [B,3,H,W], boxes int32 [n,4] as (x0,y0,x1,y1)
    half-open pixel rectangles, tier uint8 [n], box_offsets int32 [B+1],
    frac float64 [B] = the critical-area fraction each frame was drawn for,
    NaN where the rule has none).
    """
    H, W = cfg.H, cfg.W
    images = np.empty((cfg.B, 3, H, W), dtype=np.float32)
    boxes, tiers, offs, fracs = [], [], [0], []
    for i in range(cfg.B):
        rng = np.random.default_rng(1000 * seed + i)
        frac = float("nan")
        if cfg.box_rule == "single48":
            img = rng.uniform(0.0, 1.0, size=(3, H, W)).astype(np.float32)
            x0 = int(rng.integers(0, W - 48 + 1))
            y0 = int(rng.integers(0, H - 48 + 1))
            bx, tr = [(x0, y0, x0 + 48, y0 + 48)], [cfg.n_levels - 1]
        else:
            rects = [_rand_box(rng, H, W, cfg.side_lo, cfg.side_hi) for _ in range(20)]
            img = _paint_frame(rng, cfg, rects)
            if cfg.box_rule == "poisson":
                n = int(np.clip(rng.poisson(cfg.box_lambda), 1, 20))
                bx, tr = rects[:n], [cfg.n_levels - 1] * n
            elif cfg.box_rule == "fraction":
                # Boxes (painted rectangles first, then fresh draws) are added
                # until the union of their pixels reaches the drawn fraction.
                frac = float(rng.uniform(cfg.frac_lo, cfg.frac_hi))
                mask = np.zeros((H, W), dtype=bool)
                bx, k = [], 0
                while mask.mean() < frac and k < 4000:
                    b = rects[k] if k < len(rects) else _rand_box(
                        rng, H, W, cfg.side_lo, cfg.side_hi)
                    mask[b[1]:b[3], b[0]:b[2]] = True
                    bx.append(b)
                    k += 1
                tr = [cfg.n_levels - 1] * len(bx)
            elif cfg.box_rule == "tiered":
                n = int(max(1, rng.poisson(cfg.box_lambda)))
                bx = [rects[k] if k < len(rects) else _rand_box(
                    rng, H, W, cfg.side_lo, cfg.side_hi) for k in range(n)]
                u = rng.uniform(0.0, 1.0, size=n)
                top = cfg.n_levels - 1
                tr = [top if x < 0.3 else (max(top - 1, 0) if x < 0.7 else 0) for x in u]
            else:
                raise ValueError(cfg.box_rule)
        images[i] = img
        boxes.extend(bx)
        tiers.extend(tr)
        offs.append(len(boxes))
        fracs.append(frac)
    if cfg.image_dtype == "bf16":
        images = bf16_round(images)
    return (images,
            np.asarray(boxes, dtype=np.int32).reshape(-1, 4),
            np.asarray(tiers, dtype=np.uint8),
            np.asarray(offs, dtype=np.int32),
            np.asarray(fracs, dtype=np.float64))


def make_workload(cfg_or_id, seed: Optional[int] = None, sharp: bool = False) -> dict:
    """One full workload: frames, boxes, tiers and weights for a config."""
    if isinstance(cfg_or_id, int):
        cfg, cid = CONFIGS[cfg_or_id], cfg_or_id
    else:
        cfg, cid = cfg_or_id, 0
    if seed is None:
        seed = cid
    images, boxes, tier, box_offsets, frac = make_frames(cfg, seed)
    return {
        "cfg": cfg, "seed": seed, "images": images, "boxes": boxes, "tier": tier,
        "box_offsets": box_offsets, "frac": frac,
        "weights": make_weights(cfg, 7 + seed, sharp=sharp),
    }


def make_queries(cfg: Config, seed: int, n_queries: int = 128, easy_frames=()) -> np.ndarray:
    """Object queries of the coarse stage for every frame, float32 [B, Q, 5] =
    (cx, cy, w, h, c) with centre and size as fractions of the frame.

    Per frame: a few certain objects (c in (0.8, 1)), a Poisson number (mean 24 per 128 queries) of uncertain ones
    (c in (0.05, 0.8)) with the side law of the critical boxes, and background queries
    with c exponential around 0.01 (clipped to 0.05).  Frames listed in easy_frames get
    no uncertain query.  The values only have the shape of a detector's output; no
    detector was run."""
    B = cfg.B
    q = np.zeros((B, n_queries, 5), dtype=np.float32)
    for f in range(B):
        rng = np.random.default_rng(7000 * seed + f)
        n_hi = int(rng.integers(1, 6))
        n_mid = 0 if f in easy_frames else int(min(n_queries - n_hi, max(1, rng.poisson(24.0 * n_queries / 128))))
        kinds = np.array([2] * n_hi + [1] * n_mid + [0] * (n_queries - n_hi - n_mid))
        rng.shuffle(kinds)
        side = rng.uniform(cfg.side_lo, cfg.side_hi, (n_queries, 2))
        q[f, :, 0] = rng.uniform(0.0, 1.0, n_queries)
        q[f, :, 1] = rng.uniform(0.0, 1.0, n_queries)
        q[f, :, 2] = side[:, 0] / cfg.W
        q[f, :, 3] = side[:, 1] / cfg.H
        c = np.minimum(rng.exponential(0.01, n_queries), 0.05)
        c = np.where(kinds == 1, rng.uniform(0.0501, 0.8, n_queries), c)
        c = np.where(kinds == 2, rng.uniform(0.8001, 1.0, n_queries), c)
        q[f, :, 4] = c
    return q


def make_decoder_weights(cfg: Config, seed: int, n_queries: int = 128, layers: int = 2,
                         std: float = 0.02) -> Dict[str, np.ndarray]:
    """Random-init decoder weights (same law as make_weights): learned queries, per layer
    self-attention, cross-attention and FFN blocks, final LayerNorm, confidence and box
    heads.  Matrices are bf16-representable float32.  The query vectors and the head
    matrices are drawn wider (std 1 and 0.5) so that boxes and confidences spread over
    (0, 1) instead of sitting at 0.5."""
    rng = np.random.default_rng(90000 + seed)
    d, F, L = cfg.d, cfg.ffn, layers

    def mat(*shape, s=std):
        return bf16_round(rng.normal(0.0, s, shape).astype(np.float32))

    def vec(*shape, s=std):
        return rng.normal(0.0, s, shape).astype(np.float32)

    def gain(*shape):
        return (1.0 + rng.normal(0.0, std, shape)).astype(np.float32)

    return {
        "query_embed": rng.normal(0.0, 1.0, (n_queries, d)).astype(np.float32),
        "ln1_g": gain(L, d), "ln1_b": vec(L, d),
        "w_qkv": mat(L, 3 * d, d), "b_qkv": vec(L, 3 * d), "w_o": mat(L, d, d), "b_o": vec(L, d),
        "ln2_g": gain(L, d), "ln2_b": vec(L, d),
        "w_q": mat(L, d, d), "b_q": vec(L, d), "w_kv": mat(L, 2 * d, d), "b_kv": vec(L, 2 * d),
        "w_o2": mat(L, d, d), "b_o2": vec(L, d),
        "ln3_g": gain(L, d), "ln3_b": vec(L, d),
        "w_ff1": mat(L, F, d), "b_ff1": vec(L, F), "w_ff2": mat(L, d, F), "b_ff2": vec(L, d),
        "lnf_g": gain(d), "lnf_b": vec(d),
        "w_cls": mat(1, d, s=0.5), "b_cls": vec(1, s=0.5),
        "w_box1": mat(d, d, s=0.1), "b_box1": vec(d), "w_box2": mat(d, d, s=0.1), "b_box2": vec(d),
        "w_box3": mat(4, d, s=0.5), "b_box3": vec(4, s=0.5),
    }
