"""ctypes binding of include/realb.h: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

BF16, FP4, FORCE_NONE = 0, 1, -1
_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = [
    "realb_default_config", "realb_create", "realb_destroy", "realb_last_error", "realb_get_M", "realb_set_M",
    "realb_route_stats", "realb_select_precision", "realb_select_precision_host", "realb_quantize_experts_fp4",
    "realb_quantize_rows_fp4", "realb_permute", "realb_grouped_moe_ffn", "realb_grouped_moe_ffn_gate_up",
    "realb_grouped_moe_ffn_down", "realb_set_gemm_tile", "realb_combine", "realb_layer_forward", "realb_rank_forward",
    "realb_quantize_rows_nvfp4", "realb_amax_bf16", "realb_route_stats_static",
    "realb_workspace_bytes", "realb_scale_offset", "realb_scale_index_map", "realb_prefetch_join", "realb_stage_timing", "realb_stage_ms",
]


class RealbError(RuntimeError):
    pass


class Config(C.Structure):
    _fields_ = [("T_max", C.c_int), ("E", C.c_int), ("k", C.c_int), ("D", C.c_int), ("H", C.c_int), ("I", C.c_int),
                ("C", C.c_double), ("tau", C.c_double), ("M_init", C.c_double), ("aimd_mul", C.c_double),
                ("aimd_add", C.c_double), ("Gamma", C.c_longlong), ("aimd_enabled", C.c_int), ("update_first", C.c_int)]


class LayerIO(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("is_vision", C.c_void_p), ("x", C.c_void_p), ("T", C.c_int),
                ("w13", C.c_void_p), ("w2", C.c_void_p), ("rank", C.c_int), ("force", C.c_int), ("overlap", C.c_int),
                ("max_rows", C.c_longlong),
                ("next_w13", C.c_void_p), ("next_w2", C.c_void_p), ("next_w13_q", C.c_void_p), ("next_w13_s", C.c_void_p),
                ("next_w2_q", C.c_void_p), ("next_w2_s", C.c_void_p), ("reserve_cus", C.c_int),
                ("topk_ids", C.c_void_p), ("topk_w", C.c_void_p), ("expert_cnt", C.c_void_p), ("expert_vis", C.c_void_p),
                ("rank_load", C.c_void_p), ("rank_vis", C.c_void_p),
                ("expert_offsets", C.c_void_p), ("row_to_assign", C.c_void_p), ("assign_to_row", C.c_void_p),
                ("x_perm", C.c_void_p), ("x_q", C.c_void_p), ("x_s", C.c_void_p),
                ("w13_q", C.c_void_p), ("w13_s", C.c_void_p), ("w2_q", C.c_void_p), ("w2_s", C.c_void_p),
                ("h_mid", C.c_void_p), ("h_s", C.c_void_p), ("y_rows", C.c_void_p), ("out", C.c_void_p),
                ("prec_host", C.c_int32 * 64), ("ib_global", C.c_double), ("M_after", C.c_double)]


def library_path() -> str:
    return os.path.join(_PKG, "librealb.so")


def load_library() -> C.CDLL:
    """Loads librealb.so from the package directory; raises if it is not built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RealbError(f"{path} is missing: run `python -m paper_2604_19503_amd.build` (or __graft_entry__.build()) first")
    lib = C.CDLL(path)
    for name in EXPORTS:
        if not hasattr(lib, name):
            raise RealbError(f"{path} does not export {name}")
    lib.realb_last_error.restype = C.c_char_p
    lib.realb_get_M.restype = C.c_double
    lib.realb_get_M.argtypes = [C.c_void_p]
    lib.realb_set_M.argtypes = [C.c_void_p, C.c_double]
    lib.realb_default_config.restype = None
    lib.realb_default_config.argtypes = [C.POINTER(Config)] + [C.c_int] * 6
    lib.realb_workspace_bytes.restype = C.c_size_t
    lib.realb_workspace_bytes.argtypes = [C.POINTER(Config)]
    lib.realb_scale_offset.restype = C.c_size_t
    lib.realb_scale_offset.argtypes = [C.c_longlong, C.c_int, C.c_int]
    lib.realb_scale_index_map.argtypes = [C.c_longlong, C.c_int, C.c_void_p]
    lib.realb_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
    lib.realb_destroy.argtypes = [C.c_void_p]
    vp = C.c_void_p
    lib.realb_route_stats.argtypes = [vp, vp, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp]
    lib.realb_route_stats_static.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, vp]
    lib.realb_select_precision.argtypes = [vp, vp, vp, C.c_int, C.c_int, vp, vp, vp, vp]
    lib.realb_select_precision_host.argtypes = [C.POINTER(Config), vp, vp, C.c_int, C.c_int, vp, vp, vp]
    lib.realb_quantize_experts_fp4.argtypes = [vp, vp, vp, C.c_int, vp, vp, vp, vp, vp]
    lib.realb_quantize_rows_fp4.argtypes = [vp, C.c_longlong, C.c_int, vp, vp, vp]
    lib.realb_permute.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_longlong, vp, vp, vp, vp, vp, vp, vp]
    lib.realb_grouped_moe_ffn.argtypes = [vp, C.c_int, vp, C.c_int, C.c_longlong, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.realb_grouped_moe_ffn_gate_up.argtypes = [vp, C.c_int, vp, C.c_int, C.c_longlong, vp, vp, vp, vp, vp, vp, vp]
    lib.realb_grouped_moe_ffn_down.argtypes = [vp, C.c_int, vp, C.c_int, C.c_longlong, vp, vp, vp, vp, vp, vp]
    lib.realb_combine.argtypes = [vp, vp, vp, vp, C.c_int, vp, vp]
    lib.realb_layer_forward.argtypes = [vp, C.POINTER(LayerIO), vp]
    lib.realb_rank_forward.argtypes = [vp, C.POINTER(LayerIO), C.c_int, vp]
    lib.realb_prefetch_join.argtypes = [vp, vp]
    lib.realb_stage_timing.argtypes = [vp, C.c_int]
    lib.realb_stage_ms.argtypes = [vp, vp]
    lib.realb_quantize_rows_nvfp4.argtypes = [vp, C.c_longlong, C.c_int, C.c_float, vp, vp, vp]
    lib.realb_amax_bf16.argtypes = [vp, C.c_longlong, vp, vp]
    _LIB = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise RealbError(f"realb error {rc}: {load_library().realb_last_error().decode()}")


def _p(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return C.c_void_p(t.data_ptr())
    return t


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def bf16_from_bits(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy uint16 bf16 patterns -> torch.bfloat16 tensor on the device."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def scale_index_map(rows: int, K: int) -> np.ndarray:
    """realb_scale_index_map: int64 [rows, K/32] byte offsets into a K-step-tiled scale tensor."""
    idx = np.empty((rows, K // 32), dtype=np.int64)
    _check(load_library().realb_scale_index_map(rows, K, idx.ctypes.data))
    return idx


def workspace_bytes(cfg: Config) -> int:
    return int(load_library().realb_workspace_bytes(C.byref(cfg)))


def scales_to_canonical(s, rows: int, K: int) -> np.ndarray:
    """Pure index permutation (no arithmetic): a K-step-tiled scale tensor, as the library reads
    and writes it, rearranged to the plain [rows, K/32] order through the library's own index map."""
    flat = (s.detach().cpu().numpy() if isinstance(s, torch.Tensor) else np.asarray(s)).reshape(-1)
    return flat[scale_index_map(rows, K)]


def bits_from_bf16(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def set_gemm_tile(wn: int):
    _check(load_library().realb_set_gemm_tile(int(wn)))


def default_config(T_max, E, k, D, H, I) -> Config:
    cfg = Config()
    load_library().realb_default_config(C.byref(cfg), T_max, E, k, D, H, I)
    return cfg


def select_precision_host(cfg: Config, rank_load, rank_vis, T: int, M: float, force: int = FORCE_NONE):
    """realb_select_precision_host: returns (prec[D], ib_global, M_after).  No GPU."""
    load = np.ascontiguousarray(rank_load, dtype=np.int32)
    vis = np.ascontiguousarray(rank_vis, dtype=np.int32)
    prec = np.zeros(cfg.D, dtype=np.int32)
    Mio, ib = C.c_double(M), C.c_double(0)
    _check(load_library().realb_select_precision_host(C.byref(cfg), load.ctypes.data, vis.ctypes.data, T, force,
                                                      C.addressof(Mio), prec.ctypes.data, C.addressof(ib)))
    return prec, ib.value, Mio.value


def quantize_rows_fp4(x: torch.Tensor, stream=None):
    """realb_quantize_rows_fp4 on a bf16 [rows,K] tensor -> (q u8 [rows,K/2], s u8 K-step-tiled,
    ceil(rows/32)*32 * K/32 bytes; see scales_to_canonical)."""
    rows, K = x.shape
    q = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    s = torch.zeros((-(-rows // 32) * 32, K // 32), dtype=torch.uint8, device=x.device)
    _check(load_library().realb_quantize_rows_fp4(_p(x), rows, K, _p(q), _p(s), _stream(stream)))
    return q, s


def amax_bf16(x: torch.Tensor, stream=None) -> torch.Tensor:
    """realb_amax_bf16: max |x| of a bf16 tensor (element count a multiple of 8) as a 1-element float tensor."""
    out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(load_library().realb_amax_bf16(_p(x), x.numel(), _p(out), _stream(stream)))
    return out


def quantize_rows_nvfp4(x: torch.Tensor, global_scale: float, stream=None):
    """realb_quantize_rows_nvfp4 on a bf16 [rows,K] tensor -> (q u8 [rows,K/2], s u8 [rows,K/16] E4M3 bytes)."""
    rows, K = x.shape
    q = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    s = torch.empty((rows, K // 16), dtype=torch.uint8, device=x.device)
    _check(load_library().realb_quantize_rows_nvfp4(_p(x), rows, K, C.c_float(global_scale), _p(q), _p(s), _stream(stream)))
    return q, s


def route_stats_static(logits, is_vision, E: int, k: int, D: int, b, T=None, stream=None):
    """realb_route_stats_static: the routing call that allocates nothing and needs no context; writes into
    the caller's buffers b (topk_ids, topk_w, expert_cnt, expert_vis, rank_load, rank_vis)."""
    T = logits.shape[0] if T is None else T
    _check(load_library().realb_route_stats_static(_p(logits), _p(is_vision), T, E, k, D, _p(b.topk_ids), _p(b.topk_w),
                                                   _p(b.expert_cnt), _p(b.expert_vis), _p(b.rank_load), _p(b.rank_vis),
                                                   _stream(stream)))


class LayerBuffers:
    """Caller-side allocation of every tensor of one layer call (device memory via torch)."""

    def __init__(self, cfg: Config, T: int, device="cuda"):
        E, k, D, H, I = cfg.E, cfg.k, cfg.D, cfg.H, cfg.I
        nl = E // D
        self.T, self.n_local = T, nl
        self.max_rows = max(1, T * min(k, nl))
        R = self.max_rows
        dev = device
        i32 = dict(dtype=torch.int32, device=dev)
        u8 = dict(dtype=torch.uint8, device=dev)
        bf = dict(dtype=torch.bfloat16, device=dev)
        self.topk_ids = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.expert_cnt = torch.empty(E, **i32)
        self.expert_vis = torch.empty(E, **i32)
        self.rank_load = torch.empty(D, **i32)
        self.rank_vis = torch.empty(D, **i32)
        self.expert_offsets = torch.empty(nl + 1, **i32)
        self.row_to_assign = torch.empty(R, **i32)
        self.assign_to_row = torch.empty(max(1, T * k), **i32)
        self.x_perm = torch.empty((R, H), **bf)
        self.x_q = torch.empty((R, H // 2), **u8)
        R32 = -(-R // 32) * 32                           # scale tensors cover whole groups of 32 rows
        self.x_s = torch.empty((R32, H // 32), **u8)
        self.w13_q = torch.empty((nl, 2 * I, H // 2), **u8)
        self.w13_s = torch.empty((nl, 2 * I, H // 32), **u8)
        self.w2_q = torch.empty((nl, H, I // 2), **u8)
        self.w2_s = torch.empty((nl, H, I // 32), **u8)
        self.h_mid = torch.empty((R, I), **bf)          # FP4 path uses its first R*I/2 bytes as codes
        self.h_s = torch.empty((R32, I // 32), **u8)
        self.y_rows = torch.empty((R, H), **bf)
        self.out = torch.empty((T, H), **bf)


class WeightBuffers:
    """One set of FP4 weight buffers (codes and K-step-tiled scales) for a rank's experts; two of them
    serve the cross-layer prefetch as a ping-pong pair."""

    def __init__(self, cfg: Config, device="cuda"):
        nl, H, I = cfg.E // cfg.D, cfg.H, cfg.I
        u8 = dict(dtype=torch.uint8, device=device)
        self.w13_q = torch.empty((nl, 2 * I, H // 2), **u8)
        self.w13_s = torch.empty((nl, 2 * I, H // 32), **u8)
        self.w2_q = torch.empty((nl, H, I // 2), **u8)
        self.w2_s = torch.empty((nl, H, I // 32), **u8)


class Context:
    """Owns a realb_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, cfg: Config):
        self.lib = load_library()
        self.cfg = cfg
        self._h = C.c_void_p()
        _check(self.lib.realb_create(C.byref(cfg), C.byref(self._h)))

    def close(self):
        if self._h:
            self.lib.realb_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def M(self) -> float:
        return self.lib.realb_get_M(self._h)

    @M.setter
    def M(self, v: float):
        _check(self.lib.realb_set_M(self._h, float(v)))

    def route_stats(self, logits, is_vision, b: LayerBuffers, stream=None):
        _check(self.lib.realb_route_stats(self._h, _p(logits), _p(is_vision), logits.shape[0], _p(b.topk_ids), _p(b.topk_w),
                                          _p(b.expert_cnt), _p(b.expert_vis), _p(b.rank_load), _p(b.rank_vis), _stream(stream)))

    def select_precision(self, b: LayerBuffers, T: int, force: int = FORCE_NONE, stream=None):
        prec = np.zeros(self.cfg.D, dtype=np.int32)
        ib, M = C.c_double(0), C.c_double(0)
        _check(self.lib.realb_select_precision(self._h, _p(b.rank_load), _p(b.rank_vis), T, force, prec.ctypes.data,
                                               C.addressof(ib), C.addressof(M), _stream(stream)))
        return prec, ib.value, M.value

    def quantize_experts_fp4(self, w13, w2, b: LayerBuffers, stream=None):
        _check(self.lib.realb_quantize_experts_fp4(self._h, _p(w13), _p(w2), w13.shape[0], _p(b.w13_q), _p(b.w13_s),
                                                   _p(b.w2_q), _p(b.w2_s), _stream(stream)))

    def permute(self, x, b: LayerBuffers, rank: int, prec: int, stream=None):
        _check(self.lib.realb_permute(self._h, _p(x), _p(b.topk_ids), x.shape[0], rank, prec, b.max_rows,
                                      _p(b.expert_offsets), _p(b.row_to_assign), _p(b.assign_to_row),
                                      _p(b.x_perm), _p(b.x_q), _p(b.x_s), _stream(stream)))

    def grouped_moe_ffn(self, prec: int, w13, w2, b: LayerBuffers, stream=None):
        if prec == FP4:
            args = (_p(b.x_q), _p(b.x_s), _p(b.w13_q), _p(b.w13_s), _p(b.w2_q), _p(b.w2_s))
        else:
            args = (_p(b.x_perm), None, _p(w13), None, _p(w2), None)
        _check(self.lib.realb_grouped_moe_ffn(self._h, prec, _p(b.expert_offsets), b.n_local, b.max_rows, *args,
                                              _p(b.h_mid), _p(b.h_s), _p(b.y_rows), _stream(stream)))

    def grouped_moe_ffn_gate_up(self, prec: int, w13, b: LayerBuffers, stream=None):
        args = (_p(b.x_q), _p(b.x_s), _p(b.w13_q), _p(b.w13_s)) if prec == FP4 else (_p(b.x_perm), None, _p(w13), None)
        _check(self.lib.realb_grouped_moe_ffn_gate_up(self._h, prec, _p(b.expert_offsets), b.n_local, b.max_rows, *args,
                                                      _p(b.h_mid), _p(b.h_s), _stream(stream)))

    def grouped_moe_ffn_down(self, prec: int, w2, b: LayerBuffers, stream=None):
        args = (_p(b.w2_q), _p(b.w2_s)) if prec == FP4 else (_p(w2), None)
        _check(self.lib.realb_grouped_moe_ffn_down(self._h, prec, _p(b.expert_offsets), b.n_local, b.max_rows,
                                                   _p(b.h_mid), _p(b.h_s), *args, _p(b.y_rows), _stream(stream)))

    def combine(self, b: LayerBuffers, stream=None):
        _check(self.lib.realb_combine(self._h, _p(b.y_rows), _p(b.assign_to_row), _p(b.topk_w), b.T, _p(b.out), _stream(stream)))

    def make_io(self, logits, is_vision, x, w13, w2, b: LayerBuffers, rank: int, force: int = FORCE_NONE,
                overlap=True) -> LayerIO:
        """overlap: 0/False = weight encoding on the call's stream, 1/True = on the context's side stream,
        2 = skipped (the buffers already hold this layer's encoded weights), 3 = speculative (before routing),
        4 = prefetched by the previous call (see set_prefetch)."""
        io = LayerIO()
        g = lambda t: None if t is None else t.data_ptr()
        io.logits, io.is_vision, io.x, io.T = g(logits), g(is_vision), g(x), x.shape[0]
        io.w13, io.w2, io.rank, io.force, io.overlap, io.max_rows = g(w13), g(w2), rank, force, int(overlap), b.max_rows
        for name in ("topk_ids", "topk_w", "expert_cnt", "expert_vis", "rank_load", "rank_vis", "expert_offsets",
                     "row_to_assign", "assign_to_row", "x_perm", "x_q", "x_s", "w13_q", "w13_s", "w2_q", "w2_s",
                     "h_mid", "h_s", "y_rows", "out"):
            setattr(io, name, getattr(b, name).data_ptr())
        io._keep = (logits, is_vision, x, w13, w2, b)
        return io

    def layer_forward(self, io: LayerIO, stream=None):
        _check(self.lib.realb_layer_forward(self._h, C.byref(io), _stream(stream)))
        return int(io.prec_host[io.rank])

    def set_prefetch(self, io: LayerIO, next_w13, next_w2, wbuf: "WeightBuffers", reserve_cus: int):
        """Arms the cross-layer prefetch of a layer call: the next layer's weights are encoded into wbuf beside
        this layer's GEMMs, which leave reserve_cus compute units free."""
        io.next_w13, io.next_w2 = next_w13.data_ptr(), next_w2.data_ptr()
        io.next_w13_q, io.next_w13_s, io.next_w2_q, io.next_w2_s = (t.data_ptr() for t in (wbuf.w13_q, wbuf.w13_s, wbuf.w2_q, wbuf.w2_s))
        io.reserve_cus = int(reserve_cus)
        io._keep_next = (next_w13, next_w2, wbuf)

    def use_weight_buffers(self, io: LayerIO, wbuf: "WeightBuffers"):
        """Points a layer call's FP4 weight buffers at wbuf (instead of the LayerBuffers' own)."""
        io.w13_q, io.w13_s, io.w2_q, io.w2_s = (t.data_ptr() for t in (wbuf.w13_q, wbuf.w13_s, wbuf.w2_q, wbuf.w2_s))
        io._keep_w = wbuf

    STAGES = ("route_stats", "permute_indices", "decision_and_encode", "gather", "gate_up", "down", "combine")

    def stage_timing(self, enable: bool):
        _check(self.lib.realb_stage_timing(self._h, int(bool(enable))))

    def stage_ms(self) -> dict:
        """realb_stage_ms: GPU milliseconds of each stage of the last layer call (waits for it)."""
        ms = (C.c_float * len(self.STAGES))()
        _check(self.lib.realb_stage_ms(self._h, ms))
        return dict(zip(self.STAGES, (float(v) for v in ms)))

    def prefetch_join(self, stream=None):
        _check(self.lib.realb_prefetch_join(self._h, _stream(stream)))

    def rank_forward(self, io: LayerIO, prec: int, stream=None):
        _check(self.lib.realb_rank_forward(self._h, C.byref(io), prec, _stream(stream)))
