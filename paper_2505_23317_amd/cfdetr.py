"""ctypes binding over libcfdetr.so (argument marshalling only).

The functions ``cfdetr_*`` mirror the C ABI declared in include/cfdetr.h one to
one and take raw device addresses.  ``Encoder`` is a small convenience wrapper
that keeps the weights on the device as torch tensors and passes their
addresses; every step of the computation runs in the library's HIP kernels.
PyTorch is used for device memory and streams only.

There is no fallback: if the shared library has not been built, importing any
entry point raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcfdetr.so")

CFDETR_OK, CFDETR_EINVAL, CFDETR_ESHAPE, CFDETR_ECAPACITY, CFDETR_ENOMEM, CFDETR_EDEVICE = range(6)
CFDETR_BF16, CFDETR_FP32 = 0, 1
CFDETR_MAX_LEVELS = 3
KERNEL_NAMES = ["select", "plan", "embed", "gather", "layernorm", "qkv", "attention",
                "out_proj", "ffn1", "ffn2", "roi", "dec"]
CFDETR_K_COUNT = len(KERNEL_NAMES)
STATUS_NAMES = ["OK", "EINVAL", "ESHAPE", "ECAPACITY", "ENOMEM", "EDEVICE"]

EXPORTS = [
    "cfdetr_create", "cfdetr_destroy", "cfdetr_last_error", "cfdetr_workspace_bytes",
    "cfdetr_sync_status", "cfdetr_coarse_encode", "cfdetr_propose_rois", "cfdetr_select_fine",
    "cfdetr_select_fine_hard", "cfdetr_select_fine_static",
    "cfdetr_fine_encode", "cfdetr_fine_encode_padded",
    "cfdetr_multilevel_batch", "cfdetr_profile_begin", "cfdetr_profile_end",
    "cfdetr_sched_response_times", "cfdetr_sched_coarse_batch", "cfdetr_sched_fine_batches",
    "cfdetr_sched_decide", "cfdetr_decoder_attach", "cfdetr_decode", "cfdetr_merge_detections",
]
POLICIES = {"C": 0, "CF": 1, "[C]F": 2, "C[F]": 3, "[C][F]": 4}
SCHED_ACTIONS = ["idle", "coarse", "fine"]


class CfdetrConfig(ctypes.Structure):
    _fields_ = [
        ("n_levels", ctypes.c_int32),
        ("patch", ctypes.c_int32 * CFDETR_MAX_LEVELS),
        ("img_h", ctypes.c_int32), ("img_w", ctypes.c_int32),
        ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
        ("n_layers", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
        ("max_batch", ctypes.c_int32), ("max_tokens_total", ctypes.c_int32),
        ("image_dtype", ctypes.c_int), ("act_dtype", ctypes.c_int),
        ("ln_eps", ctypes.c_float),
    ]


class CfdetrRoiParams(ctypes.Structure):
    _fields_ = [("tau_hi", ctypes.c_float), ("tau_lo", ctypes.c_float),
                ("scale", ctypes.c_float), ("min_side", ctypes.c_float),
                ("tier", ctypes.c_int32)]


class CfdetrWeights(ctypes.Structure):
    _fields_ = [
        ("w_embed", ctypes.c_void_p * CFDETR_MAX_LEVELS),
        ("b_embed", ctypes.c_void_p * CFDETR_MAX_LEVELS),
        ("ln1_g", ctypes.c_void_p), ("ln1_b", ctypes.c_void_p),
        ("w_qkv", ctypes.c_void_p), ("b_qkv", ctypes.c_void_p),
        ("w_o", ctypes.c_void_p), ("b_o", ctypes.c_void_p),
        ("ln2_g", ctypes.c_void_p), ("ln2_b", ctypes.c_void_p),
        ("w_ff1", ctypes.c_void_p), ("b_ff1", ctypes.c_void_p),
        ("w_ff2", ctypes.c_void_p), ("b_ff2", ctypes.c_void_p),
        ("lnf_g", ctypes.c_void_p), ("lnf_b", ctypes.c_void_p),
    ]


DECODER_MATRICES = ("w_qkv", "w_o", "w_q", "w_kv", "w_o2", "w_ff1", "w_ff2", "w_cls", "w_box1",
                    "w_box2", "w_box3")
DECODER_FIELDS = ("query_embed", "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
                  "w_q", "b_q", "w_kv", "b_kv", "w_o2", "b_o2", "ln3_g", "ln3_b", "w_ff1", "b_ff1",
                  "w_ff2", "b_ff2", "lnf_g", "lnf_b", "w_cls", "b_cls", "w_box1", "b_box1",
                  "w_box2", "b_box2", "w_box3", "b_box3")


class CfdetrDecoderWeights(ctypes.Structure):
    _fields_ = ([("n_queries", ctypes.c_int32), ("n_layers", ctypes.c_int32)]
                + [(name, ctypes.c_void_p) for name in DECODER_FIELDS])


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libcfdetr.so and declare the prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2505_23317_amd.build); "
            "there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    lib.cfdetr_create.argtypes = [ctypes.POINTER(CfdetrConfig), ctypes.POINTER(CfdetrWeights),
                                  ctypes.POINTER(vp)]
    lib.cfdetr_create.restype = ctypes.c_int
    lib.cfdetr_destroy.argtypes = [vp]
    lib.cfdetr_destroy.restype = None
    lib.cfdetr_last_error.argtypes = [vp]
    lib.cfdetr_last_error.restype = ctypes.c_char_p
    lib.cfdetr_workspace_bytes.argtypes = [vp]
    lib.cfdetr_workspace_bytes.restype = ctypes.c_uint64
    lib.cfdetr_sync_status.argtypes = [vp, vp]
    lib.cfdetr_sync_status.restype = ctypes.c_int
    lib.cfdetr_coarse_encode.argtypes = [vp, vp, i32, vp, vp, vp]
    lib.cfdetr_coarse_encode.restype = ctypes.c_int
    lib.cfdetr_propose_rois.argtypes = [vp, vp, i32, i32, ctypes.POINTER(CfdetrRoiParams), i32,
                                        vp, vp, vp, vp, vp, vp]
    lib.cfdetr_propose_rois.restype = ctypes.c_int
    lib.cfdetr_select_fine.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.cfdetr_select_fine.restype = ctypes.c_int
    lib.cfdetr_select_fine_hard.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.cfdetr_select_fine_hard.restype = ctypes.c_int
    lib.cfdetr_select_fine_static.argtypes = [ctypes.POINTER(CfdetrConfig), vp, vp, vp, i32, vp, vp,
                                              vp, vp, vp]
    lib.cfdetr_select_fine_static.restype = ctypes.c_int
    lib.cfdetr_fine_encode.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp]
    lib.cfdetr_fine_encode.restype = ctypes.c_int
    lib.cfdetr_fine_encode_padded.argtypes = [vp, vp, i32, vp, vp, vp, i32, vp, vp]
    lib.cfdetr_fine_encode_padded.restype = ctypes.c_int
    lib.cfdetr_multilevel_batch.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.cfdetr_multilevel_batch.restype = ctypes.c_int
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
    dbl = ctypes.c_double
    lib.cfdetr_sched_response_times.argtypes = [i32, dp, dp, dp, ip]
    lib.cfdetr_sched_response_times.restype = ctypes.c_int
    lib.cfdetr_sched_coarse_batch.argtypes = [i32, dbl, dbl, dp]
    lib.cfdetr_sched_coarse_batch.restype = i32
    lib.cfdetr_sched_fine_batches.argtypes = [i32, ip, dp, dbl, dbl, dp, i32, i32, ip, ip, ip, dp]
    lib.cfdetr_sched_fine_batches.restype = ctypes.c_int
    lib.cfdetr_sched_decide.argtypes = [ctypes.c_int, dbl, i32, ip, i32, ip, ip, dp, dbl, dp, dp,
                                        i32, i32, ip, ip, ip, ip]
    lib.cfdetr_sched_decide.restype = ctypes.c_int
    lib.cfdetr_merge_detections.argtypes = [vp, vp, vp, vp, i32, i32, ctypes.c_float, ctypes.c_float,
                                            vp, vp, vp, vp]
    lib.cfdetr_merge_detections.restype = ctypes.c_int
    lib.cfdetr_decoder_attach.argtypes = [vp, ctypes.POINTER(CfdetrDecoderWeights)]
    lib.cfdetr_decoder_attach.restype = ctypes.c_int
    lib.cfdetr_decode.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.cfdetr_decode.restype = ctypes.c_int
    lib.cfdetr_profile_begin.argtypes = [vp]
    lib.cfdetr_profile_begin.restype = ctypes.c_int
    lib.cfdetr_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float),
                                       ctypes.POINTER(ctypes.c_int32)]
    lib.cfdetr_profile_end.restype = ctypes.c_int
    _lib = lib
    return lib


class CfdetrError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"cfdetr status {STATUS_NAMES[status] if 0 <= status < 6 else status}"
                         f": {message}")
        self.status = status


def _check(status: int, ctx=None):
    if status != CFDETR_OK:
        raw = load_library().cfdetr_last_error(ctx)
        msg = raw.decode() if raw else ""
        raise CfdetrError(status, msg)


# ---- one-to-one wrappers (raw addresses in, status checked) -----------------
def cfdetr_create(cfg: CfdetrConfig, weights: CfdetrWeights) -> int:
    out = ctypes.c_void_p()
    _check(load_library().cfdetr_create(ctypes.byref(cfg), ctypes.byref(weights),
                                        ctypes.byref(out)))
    return out.value


def cfdetr_destroy(ctx: int) -> None:
    load_library().cfdetr_destroy(ctx)


def cfdetr_last_error(ctx: int) -> str:
    raw = load_library().cfdetr_last_error(ctx)
    return raw.decode() if raw else ""


def cfdetr_workspace_bytes(ctx: int) -> int:
    return int(load_library().cfdetr_workspace_bytes(ctx))


def cfdetr_sync_status(ctx: int, stream: int = 0) -> None:
    _check(load_library().cfdetr_sync_status(ctx, stream), ctx)


def cfdetr_coarse_encode(ctx, images, B, x0_cache, y_coarse, stream=0) -> None:
    _check(load_library().cfdetr_coarse_encode(ctx, images, B, x0_cache, y_coarse, stream), ctx)


def cfdetr_propose_rois(ctx, queries, B, Q, params: CfdetrRoiParams, max_boxes, boxes, tier,
                        box_offsets, hard, mean_conf, stream=0) -> None:
    _check(load_library().cfdetr_propose_rois(ctx, queries, B, Q, ctypes.byref(params), max_boxes,
                                              boxes, tier, box_offsets, hard, mean_conf, stream),
           ctx)


def cfdetr_merge_detections(ctx, coarse, fine, hard, B, Q, tau_hi, tau_fine, det, src, count,
                            stream=0) -> None:
    _check(load_library().cfdetr_merge_detections(ctx, coarse, fine, hard, B, Q, tau_hi, tau_fine,
                                                  det, src, count, stream), ctx)


def cfdetr_decoder_attach(ctx, weights: CfdetrDecoderWeights) -> None:
    _check(load_library().cfdetr_decoder_attach(ctx, ctypes.byref(weights)), ctx)


def cfdetr_decode(ctx, memory, cu_seqlens, B, queries, stream=0) -> None:
    _check(load_library().cfdetr_decode(ctx, memory, cu_seqlens, B, queries, stream), ctx)


def cfdetr_select_fine(ctx, boxes, tier, box_offsets, B, tok_desc, cu_seqlens, level_counts,
                       stream=0) -> None:
    _check(load_library().cfdetr_select_fine(ctx, boxes, tier, box_offsets, B, tok_desc,
                                             cu_seqlens, level_counts, stream), ctx)


def cfdetr_select_fine_hard(ctx, boxes, tier, box_offsets, hard, B, tok_desc, cu_seqlens,
                            level_counts, stream=0) -> None:
    _check(load_library().cfdetr_select_fine_hard(ctx, boxes, tier, box_offsets, hard, B, tok_desc,
                                                  cu_seqlens, level_counts, stream), ctx)


def cfdetr_select_fine_static(cfg: CfdetrConfig, boxes, tier, box_offsets, B, tok_desc, cu_seqlens,
                              level_counts, overflow, stream=0) -> None:
    _check(load_library().cfdetr_select_fine_static(ctypes.byref(cfg), boxes, tier, box_offsets, B,
                                                    tok_desc, cu_seqlens, level_counts, overflow,
                                                    stream), None)


def cfdetr_fine_encode(ctx, images, B, tok_desc, cu_seqlens, x0_cache, y_mixed, stream=0) -> None:
    _check(load_library().cfdetr_fine_encode(ctx, images, B, tok_desc, cu_seqlens, x0_cache,
                                             y_mixed, stream), ctx)


def cfdetr_fine_encode_padded(ctx, images, B, tok_desc, cu_seqlens, x0_cache, t_pad, y_padded,
                              stream=0) -> None:
    _check(load_library().cfdetr_fine_encode_padded(ctx, images, B, tok_desc, cu_seqlens, x0_cache,
                                                    t_pad, y_padded, stream), ctx)


def cfdetr_multilevel_batch(ctx, images, B, boxes, tier, box_offsets, y_coarse, y_mixed,
                            tok_desc, cu_seqlens, level_counts, stream=0) -> None:
    _check(load_library().cfdetr_multilevel_batch(ctx, images, B, boxes, tier, box_offsets,
                                                  y_coarse, y_mixed, tok_desc, cu_seqlens,
                                                  level_counts, stream), ctx)


# ---- scheduling decisions (host data; lists in, lists out) ---------------------
def _darr(v):
    return (ctypes.c_double * max(len(v), 1))(*[float(x) for x in v])


def _iarr(v):
    return (ctypes.c_int32 * max(len(v), 1))(*[int(x) for x in v])


def _fine_table(c_fine):
    """[[level][size]] -> flat row-major table, n_levels, max_size."""
    n_levels, max_size = len(c_fine), len(c_fine[0]) - 1
    flat = [float(x) for row in c_fine for x in row]
    return _darr(flat), n_levels, max_size


def cfdetr_sched_response_times(period, c_coarse):
    n = len(period)
    R = (ctypes.c_double * n)()
    ok = ctypes.c_int32()
    _check(load_library().cfdetr_sched_response_times(n, _darr(period), _darr(c_coarse), R,
                                                      ctypes.byref(ok)))
    return bool(ok.value), list(R)


def cfdetr_sched_coarse_batch(n_active, t, next_release, c_batch_by_size) -> int:
    return int(load_library().cfdetr_sched_coarse_batch(n_active, t, next_release,
                                                        _darr(c_batch_by_size)))


def cfdetr_sched_fine_batches(workload, deadline, t, next_coarse_release, c_fine):
    """Returns (order, cuts, dba) like the paper's tables: cuts are half-open ranges."""
    n = len(workload)
    tab, n_levels, max_size = _fine_table(c_fine)
    order, ends = (ctypes.c_int32 * max(n, 1))(), (ctypes.c_int32 * max(n, 1))()
    nb = ctypes.c_int32()
    dba = (ctypes.c_double * (n + 1))()
    _check(load_library().cfdetr_sched_fine_batches(n, _iarr(workload), _darr(deadline), t,
                                                    next_coarse_release, tab, n_levels, max_size,
                                                    order, ends, ctypes.byref(nb), dba))
    cuts, a = [], 0
    for b in range(nb.value):
        cuts.append((a, ends[b]))
        a = ends[b]
    return list(order)[:n], cuts, list(dba)


def cfdetr_sched_decide(policy: str, t, active_coarse, active_fine, fine_workload, fine_deadline,
                        next_release, c_coarse_by_size, c_fine):
    """Returns (kind, tasks): ("coarse", [tasks]) | ("fine", [[batch], ...]) | ("idle", [])."""
    tab, n_levels, max_size = _fine_table(c_fine)
    m = max(len(active_coarse), len(active_fine), 1)
    kind, nb = ctypes.c_int32(), ctypes.c_int32()
    tasks, ends = (ctypes.c_int32 * m)(), (ctypes.c_int32 * m)()
    _check(load_library().cfdetr_sched_decide(
        POLICIES[policy], t, len(active_coarse), _iarr(active_coarse), len(active_fine),
        _iarr(active_fine), _iarr(fine_workload), _darr(fine_deadline), next_release,
        _darr(c_coarse_by_size), tab, n_levels, max_size, ctypes.byref(kind), tasks, ends,
        ctypes.byref(nb)))
    name = SCHED_ACTIONS[kind.value]
    if name == "coarse":
        return name, list(tasks)[:ends[0]]
    if name == "fine":
        out, a = [], 0
        for b in range(nb.value):
            out.append(list(tasks)[a:ends[b]])
            a = ends[b]
        return name, out
    return name, []


def cfdetr_profile_begin(ctx) -> None:
    _check(load_library().cfdetr_profile_begin(ctx), ctx)


def cfdetr_profile_end(ctx) -> Dict[str, Dict[str, float]]:
    ms = (ctypes.c_float * CFDETR_K_COUNT)()
    n = (ctypes.c_int32 * CFDETR_K_COUNT)()
    _check(load_library().cfdetr_profile_end(ctx, ms, n), ctx)
    return {KERNEL_NAMES[k]: {"ms": float(ms[k]), "launches": int(n[k])}
            for k in range(CFDETR_K_COUNT)}


# ---- convenience wrapper ------------------------------------------------------
def _to_device(arr: np.ndarray, as_bf16: bool):
    """numpy float32 -> torch tensor on cuda:0 (bf16 bit patterns or fp32)."""
    import torch
    from . import synth
    if as_bf16:
        bits = synth.bf16_bits(arr).view(np.int16)
        return torch.from_numpy(bits).view(torch.bfloat16).reshape(arr.shape).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()


def unpack_tok_desc(desc: np.ndarray) -> np.ndarray:
    """int32 descriptors -> [T,3] (level,row,col)."""
    d = np.asarray(desc).astype(np.int64)
    return np.stack([(d >> 28) & 7, (d >> 14) & 0x3FFF, d & 0x3FFF], axis=1)


class Encoder:
    """Device-resident weights + one library context for one model shape.

    ``cfg`` is a synth.Config (or anything with the same fields); ``weights`` a
    dict of float32 numpy arrays laid out as include/cfdetr.h describes.
    """

    def __init__(self, cfg, weights: Dict[str, np.ndarray], act_dtype: str = "bf16",
                 max_batch: Optional[int] = None, max_tokens_total: Optional[int] = None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("cfdetr needs a GPU: no CPU fallback exists")
        self.cfg = cfg
        self.act_bf16 = act_dtype == "bf16"
        self.max_batch = max_batch or cfg.B
        top = cfg.n_levels - 1
        self.max_tokens = max_tokens_total or self.max_batch * cfg.n_cells(top)
        self.n0 = cfg.n_cells(0)
        mats = {"w_qkv", "w_o", "w_ff1", "w_ff2"} | {f"w_embed{l}" for l in range(cfg.n_levels)}
        self.dev = {k: _to_device(v, self.act_bf16 and k in mats) for k, v in weights.items()}
        c = CfdetrConfig()
        c.n_levels = cfg.n_levels
        for l in range(CFDETR_MAX_LEVELS):
            c.patch[l] = cfg.patch[l] if l < cfg.n_levels else 0
        c.img_h, c.img_w = cfg.H, cfg.W
        c.d_model, c.n_heads, c.n_layers, c.d_ffn = cfg.d, cfg.heads, cfg.layers, cfg.ffn
        c.max_batch, c.max_tokens_total = self.max_batch, self.max_tokens
        c.image_dtype = CFDETR_BF16 if cfg.image_dtype == "bf16" else CFDETR_FP32
        c.act_dtype = CFDETR_BF16 if self.act_bf16 else CFDETR_FP32
        c.ln_eps = 1e-5
        w = CfdetrWeights()
        for l in range(cfg.n_levels):
            w.w_embed[l] = self.dev[f"w_embed{l}"].data_ptr()
            w.b_embed[l] = self.dev[f"b_embed{l}"].data_ptr()
        for name in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
                     "w_ff1", "b_ff1", "w_ff2", "b_ff2", "lnf_g", "lnf_b"):
            setattr(w, name, self.dev[name].data_ptr())
        self.c_cfg, self.c_w = c, w
        self.ctx = cfdetr_create(c, w)

    # -- helpers ---------------------------------------------------------------
    def upload_images(self, images: np.ndarray):
        return _to_device(images, self.cfg.image_dtype == "bf16")

    @staticmethod
    def upload_boxes(boxes, tier, box_offsets):
        import torch
        b = torch.from_numpy(np.ascontiguousarray(boxes, dtype=np.int32).reshape(-1, 4)).cuda()
        t = torch.from_numpy(np.ascontiguousarray(tier, dtype=np.uint8)).cuda()
        o = torch.from_numpy(np.ascontiguousarray(box_offsets, dtype=np.int32)).cuda()
        if b.numel() == 0:      # keep a valid address for an empty table
            b = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
            t = torch.zeros(1, dtype=torch.uint8, device="cuda")
        return b, t, o

    @staticmethod
    def _stream() -> int:
        import torch
        return torch.cuda.current_stream().cuda_stream

    def alloc_outputs(self, B: int):
        import torch
        d = self.cfg.d
        return {
            "x0_cache": torch.empty((B * self.n0, d), dtype=torch.float32, device="cuda"),
            "y_coarse": torch.empty((B * self.n0, d), dtype=torch.float32, device="cuda"),
            "y_mixed": torch.zeros((self.max_tokens, d), dtype=torch.float32, device="cuda"),
            "tok_desc": torch.zeros(self.max_tokens, dtype=torch.int32, device="cuda"),
            "cu_seqlens": torch.zeros(B + 1, dtype=torch.int32, device="cuda"),
            "level_counts": torch.zeros((B, self.cfg.n_levels), dtype=torch.int32, device="cuda"),
        }

    # -- the four calls ----------------------------------------------------------
    def coarse_encode(self, images, B, x0_cache, y_coarse):
        cfdetr_coarse_encode(self.ctx, images.data_ptr(), B,
                             x0_cache.data_ptr() if x0_cache is not None else None,
                             y_coarse.data_ptr(), self._stream())

    def propose_rois(self, queries, params: CfdetrRoiParams, boxes, tier, box_offsets, hard,
                     mean_conf):
        """queries: float32 device tensor [B, Q, 5]; the other tensors are outputs."""
        B, Q = int(queries.shape[0]), int(queries.shape[1])
        cfdetr_propose_rois(self.ctx, queries.data_ptr(), B, Q, params, int(boxes.shape[0]),
                            boxes.data_ptr(), tier.data_ptr(), box_offsets.data_ptr(),
                            hard.data_ptr(), mean_conf.data_ptr(), self._stream())

    def merge_detections(self, coarse, fine, hard, tau_hi, tau_fine, det, src, count):
        """coarse, fine: float32 device tensors [B, Q, 5]; det [B, 2Q, 5], src [B, 2Q] uint8 and
        count [B] int32 are outputs."""
        B, Q = int(coarse.shape[0]), int(coarse.shape[1])
        cfdetr_merge_detections(self.ctx, coarse.data_ptr(), fine.data_ptr(), hard.data_ptr(), B, Q,
                                tau_hi, tau_fine, det.data_ptr(), src.data_ptr(), count.data_ptr(),
                                self._stream())

    def attach_decoder(self, weights: Dict[str, np.ndarray]):
        """weights: float32 numpy arrays named as include/cfdetr.h lists them; uploaded here
        (matrices as bf16 bit patterns) and kept alive with the context."""
        self.dec_dev = {k: _to_device(v, k in DECODER_MATRICES) for k, v in weights.items()}
        w = CfdetrDecoderWeights()
        w.n_queries = int(weights["query_embed"].shape[0])
        w.n_layers = int(weights["w_qkv"].shape[0])
        for name in DECODER_FIELDS:
            setattr(w, name, self.dec_dev[name].data_ptr())
        self.n_queries = w.n_queries
        self.c_dec = w
        cfdetr_decoder_attach(self.ctx, w)

    def decode(self, memory, cu_seqlens, B, queries):
        """memory: float32 device tensor [T, d]; queries: float32 device tensor [B, Q, 5] out."""
        cfdetr_decode(self.ctx, memory.data_ptr(), cu_seqlens.data_ptr(), B, queries.data_ptr(),
                      self._stream())

    def select_fine(self, boxes, tier, box_offsets, B, tok_desc, cu_seqlens, level_counts=None):
        cfdetr_select_fine(self.ctx, boxes.data_ptr(), tier.data_ptr(), box_offsets.data_ptr(), B,
                           tok_desc.data_ptr(), cu_seqlens.data_ptr(),
                           level_counts.data_ptr() if level_counts is not None else None,
                           self._stream())

    def select_fine_hard(self, boxes, tier, box_offsets, hard, B, tok_desc, cu_seqlens,
                         level_counts=None):
        cfdetr_select_fine_hard(self.ctx, boxes.data_ptr(), tier.data_ptr(), box_offsets.data_ptr(),
                                hard.data_ptr(), B, tok_desc.data_ptr(), cu_seqlens.data_ptr(),
                                level_counts.data_ptr() if level_counts is not None else None,
                                self._stream())

    def select_fine_static(self, boxes, tier, box_offsets, B, tok_desc, cu_seqlens, level_counts,
                           overflow):
        """The selection through the entry point that allocates nothing and uses no context
        (the configuration structure of this encoder is passed instead)."""
        cfdetr_select_fine_static(self.c_cfg, boxes.data_ptr(), tier.data_ptr(),
                                  box_offsets.data_ptr(), B, tok_desc.data_ptr(),
                                  cu_seqlens.data_ptr(),
                                  level_counts.data_ptr() if level_counts is not None else None,
                                  overflow.data_ptr(), self._stream())

    def fine_encode(self, images, B, tok_desc, cu_seqlens, x0_cache, y_mixed):
        cfdetr_fine_encode(self.ctx, images.data_ptr(), B, tok_desc.data_ptr(),
                           cu_seqlens.data_ptr(),
                           x0_cache.data_ptr() if x0_cache is not None else None,
                           y_mixed.data_ptr(), self._stream())

    def fine_encode_padded(self, images, B, tok_desc, cu_seqlens, x0_cache, t_pad, y_padded):
        cfdetr_fine_encode_padded(self.ctx, images.data_ptr(), B, tok_desc.data_ptr(),
                                  cu_seqlens.data_ptr(),
                                  x0_cache.data_ptr() if x0_cache is not None else None,
                                  t_pad, y_padded.data_ptr(), self._stream())

    def multilevel_batch(self, images, B, boxes, tier, box_offsets, out):
        cfdetr_multilevel_batch(self.ctx, images.data_ptr(), B, boxes.data_ptr(), tier.data_ptr(),
                                box_offsets.data_ptr(), out["y_coarse"].data_ptr(),
                                out["y_mixed"].data_ptr(), out["tok_desc"].data_ptr(),
                                out["cu_seqlens"].data_ptr(), out["level_counts"].data_ptr(),
                                self._stream())

    def sync_status(self):
        cfdetr_sync_status(self.ctx, self._stream())

    def close(self):
        if getattr(self, "ctx", None):
            cfdetr_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
