"""Thin Python binding of libhot, the MI355X implementation of the HOT linear-layer
backward pass (arxiv 2503.21261).

Argument marshalling only: every step runs in the HIP kernels behind the C ABI
declared in ``include/hot.h``; function names here are the C names.  torch is
used for device memory and streams.  There is no CPU fallback: if the library
has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhot.so")

HOT_OK = 0
HOT_ERR_ARG, HOT_ERR_SHAPE, HOT_ERR_WORKSPACE, HOT_ERR_DEVICE, HOT_ERR_UNIMPLEMENTED = 1, 2, 3, 4, 5
HOT_ERR_SCRATCH_LIMIT = 6
HOT_NOALLOC_SCRATCH_BYTES = 64 << 20
HOT_Q_PER_TENSOR, HOT_Q_PER_TOKEN = 0, 1
HOT_ROUND_NEAREST_EVEN, HOT_ROUND_PSEUDO_STOCHASTIC = 0, 1

EXPORTS = (
    "hot_default_config", "hot_status_string", "hot_act_buffer_bytes", "hot_workspace_bytes",
    "hot_weight_buffer_bytes", "hot_gx_cached_workspace_bytes", "hot_quantize_weight", "hot_linear_backward_gx_cached",
    "hot_debug_unpack_weight", "hot_compress_activation", "hot_linear_backward_gx", "hot_linear_backward_gw",
    "hot_linear_backward", "hot_linear_backward_gx_noalloc", "hot_lowpass_l1_rows", "hot_select_quantizer", "hot_debug_unpack_activation",
    "hot_debug_gx_operands", "hot_debug_gw_operands", "hot_debug_fused_operands", "hot_debug_set_exchange_wait_us",
    "hot_debug_set_backward_strategy", "hot_debug_set_gemm_mode", "hot_debug_profile_begin", "hot_debug_profile_end", "hot_debug_profile_sequence",
    "hot_debug_stage_name", "hot_debug_probe",
)
HOT_NUM_STAGES = 15
HOT_WS_PREFIX_BYTES = 24832


class hot_config(C.Structure):
    _fields_ = [("block", C.c_int32), ("keep", C.c_int32), ("keep_idx", C.POINTER(C.c_int32)),
                ("gx_bits", C.c_int32), ("gw_bits", C.c_int32), ("rounding", C.c_int32),
                ("lqs_threshold", C.c_float), ("sample_tokens", C.c_int32), ("replayable", C.c_int32)]


class HotError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (hot_status {status})")


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Loads libhot.so; fails loudly if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_21261_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        l = C.CDLL(LIB_PATH)
        i64, vp, sz = C.c_int64, C.c_void_p, C.c_size_t
        cfgp = C.POINTER(hot_config)
        l.hot_default_config.argtypes = [cfgp]
        l.hot_default_config.restype = None
        l.hot_status_string.argtypes = [C.c_int]
        l.hot_status_string.restype = C.c_char_p
        l.hot_act_buffer_bytes.argtypes = [cfgp, i64, i64]
        l.hot_act_buffer_bytes.restype = sz
        l.hot_workspace_bytes.argtypes = [cfgp, i64, i64, i64]
        l.hot_workspace_bytes.restype = sz
        l.hot_compress_activation.argtypes = [cfgp, vp, i64, i64, vp, vp, sz, vp]
        l.hot_linear_backward_gx.argtypes = [cfgp, vp, vp, i64, i64, i64, C.c_int, vp, vp, sz, vp]
        l.hot_linear_backward_gx_noalloc.argtypes = [cfgp, vp, vp, i64, i64, i64, C.c_int, vp, vp]
        l.hot_linear_backward_gw.argtypes = [cfgp, vp, vp, i64, i64, i64, vp, vp, sz, vp]
        l.hot_linear_backward.argtypes = [cfgp, vp, vp, vp, i64, i64, i64, C.c_int, vp, vp, vp, sz, vp]
        l.hot_select_quantizer.argtypes = [cfgp, vp, i64, i64, C.POINTER(C.c_int),
                                           C.POINTER(C.c_double), C.POINTER(C.c_double), vp, sz, vp]
        l.hot_lowpass_l1_rows.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        l.hot_debug_unpack_activation.argtypes = [cfgp, vp, i64, i64, vp, vp, vp]
        l.hot_debug_gx_operands.argtypes = [cfgp, vp, i64, i64, i64, C.c_int, vp, vp, vp, vp, vp, vp]
        l.hot_debug_gw_operands.argtypes = [cfgp, vp, vp, i64, i64, i64, vp, vp, vp, vp]
        l.hot_debug_fused_operands.argtypes = [cfgp, vp, vp, i64, i64, i64, C.c_int] + [vp] * 9
        l.hot_debug_set_exchange_wait_us.argtypes = [C.c_int]
        l.hot_debug_set_backward_strategy.argtypes = [C.c_int]
        l.hot_debug_set_gemm_mode.argtypes = [C.c_int]
        l.hot_debug_profile_begin.argtypes = []
        l.hot_debug_profile_end.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_int64)]
        l.hot_debug_probe.argtypes = [C.c_int, vp, sz, C.c_int, vp]
        l.hot_debug_profile_sequence.argtypes = [C.POINTER(C.c_int32), C.c_int64]
        l.hot_weight_buffer_bytes.argtypes = [cfgp, i64, i64]
        l.hot_weight_buffer_bytes.restype = sz
        l.hot_gx_cached_workspace_bytes.argtypes = [cfgp, i64, i64, i64]
        l.hot_gx_cached_workspace_bytes.restype = sz
        l.hot_quantize_weight.argtypes = [cfgp, vp, i64, i64, vp, vp, sz, vp]
        l.hot_linear_backward_gx_cached.argtypes = [cfgp, vp, vp, i64, i64, i64, C.c_int, vp, vp, sz, vp]
        l.hot_debug_unpack_weight.argtypes = [cfgp, vp, i64, i64, vp, vp, vp]
        for name in EXPORTS[6:]:
            if name not in ("hot_debug_stage_name", "hot_debug_profile_sequence"):
                getattr(l, name).restype = C.c_int
        l.hot_debug_profile_sequence.restype = C.c_int64
        l.hot_debug_stage_name.argtypes = [C.c_int]
        l.hot_debug_stage_name.restype = C.c_char_p
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().hot_status_string(int(status)).decode()


@dataclass
class Config:
    """Python mirror of ``hot_config`` (paper defaults: n=16, r=8, INT4/INT8, PSR, 0.5)."""
    block: int = 16
    keep: int = 8
    keep_idx: Optional[Sequence[int]] = None
    gx_bits: int = 4
    gw_bits: int = 8
    rounding: int = HOT_ROUND_PSEUDO_STOCHASTIC
    lqs_threshold: float = 0.5
    sample_tokens: int = 0
    replayable: bool = False     # launch tags from the workspace epoch: calls may be recorded into a HIP graph

    def reduced_tokens(self, L: int) -> int:
        """L' = tokens after HLA: L*r/n, or B * ceil(S/n) * r with per-sample tiling."""
        if self.sample_tokens:
            return L // self.sample_tokens * (-(-self.sample_tokens // self.block)) * self.keep
        return L // self.block * self.keep

    def c(self) -> hot_config:
        cfg = hot_config()
        cfg.block, cfg.keep = int(self.block), int(self.keep)
        cfg.gx_bits, cfg.gw_bits = int(self.gx_bits), int(self.gw_bits)
        cfg.rounding, cfg.lqs_threshold = int(self.rounding), float(self.lqs_threshold)
        cfg.sample_tokens = int(self.sample_tokens)
        cfg.replayable = 1 if self.replayable else 0
        if self.keep_idx is None:
            cfg.keep_idx = None
            self._keep_arr = None
        else:
            self._keep_arr = (C.c_int32 * len(self.keep_idx))(*[int(k) for k in self.keep_idx])
            cfg.keep_idx = C.cast(self._keep_arr, C.POINTER(C.c_int32))
        return cfg


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _check(status: int, where: str) -> None:
    if status != HOT_OK:
        raise HotError(status, where)


def _dev_f32(t: torch.Tensor, shape: Tuple[int, ...], name: str) -> None:
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape):
        raise ValueError(f"{name}: expected contiguous float32 device tensor of shape {shape}")


def hot_act_buffer_bytes(cfg: Config, L: int, I: int) -> int:
    return int(lib().hot_act_buffer_bytes(C.byref(cfg.c()), L, I))


def hot_workspace_bytes(cfg: Config, L: int, O: int, I: int) -> int:
    return int(lib().hot_workspace_bytes(C.byref(cfg.c()), L, O, I))


def alloc_workspace(cfg: Config, L: int, O: int, I: int, device="cuda") -> torch.Tensor:
    n = hot_workspace_bytes(cfg, L, O, I)
    if n == 0:
        raise HotError(HOT_ERR_SHAPE, "hot_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def alloc_act_buffer(cfg: Config, L: int, I: int, device="cuda") -> torch.Tensor:
    n = hot_act_buffer_bytes(cfg, L, I)
    if n == 0:
        raise HotError(HOT_ERR_SHAPE, "hot_act_buffer_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def hot_weight_buffer_bytes(cfg: Config, O: int, I: int) -> int:
    return int(lib().hot_weight_buffer_bytes(C.byref(cfg.c()), O, I))


def hot_gx_cached_workspace_bytes(cfg: Config, L: int, O: int, I: int) -> int:
    return int(lib().hot_gx_cached_workspace_bytes(C.byref(cfg.c()), L, O, I))


def alloc_weight_buffer(cfg: Config, O: int, I: int, device="cuda") -> torch.Tensor:
    n = hot_weight_buffer_bytes(cfg, O, I)
    if n == 0:
        raise HotError(HOT_ERR_SHAPE, "hot_weight_buffer_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def hot_quantize_weight(cfg: Config, w: torch.Tensor, wq_buf: torch.Tensor, ws: torch.Tensor,
                        stream=None) -> torch.Tensor:
    O, I = w.shape
    _dev_f32(w, (O, I), "w")
    st = lib().hot_quantize_weight(C.byref(cfg.c()), _ptr(w), O, I, _ptr(wq_buf), _ptr(ws),
                                   ws.numel(), _stream(stream))
    _check(st, "hot_quantize_weight")
    return wq_buf


def hot_linear_backward_gx_cached(cfg: Config, g_y: torch.Tensor, wq_buf: torch.Tensor, I: int,
                                  gy_quantizer: int, g_x: torch.Tensor, ws: torch.Tensor,
                                  stream=None) -> torch.Tensor:
    L, O = g_y.shape
    _dev_f32(g_y, (L, O), "g_y"); _dev_f32(g_x, (L, I), "g_x")
    st = lib().hot_linear_backward_gx_cached(C.byref(cfg.c()), _ptr(g_y), _ptr(wq_buf), L, O, I,
                                             int(gy_quantizer), _ptr(g_x), _ptr(ws), ws.numel(),
                                             _stream(stream))
    _check(st, "hot_linear_backward_gx_cached")
    return g_x


def hot_debug_unpack_weight(cfg: Config, wq_buf: torch.Tensor, O: int, I: int, stream=None):
    """Returns (codes int8 [O, I], scale float32 [1]) on the device."""
    codes = torch.empty((O, I), dtype=torch.int8, device=wq_buf.device)
    scale = torch.empty(1, dtype=torch.float32, device=wq_buf.device)
    st = lib().hot_debug_unpack_weight(C.byref(cfg.c()), _ptr(wq_buf), O, I, _ptr(codes),
                                       _ptr(scale), _stream(stream))
    _check(st, "hot_debug_unpack_weight")
    return codes, scale


def hot_compress_activation(cfg: Config, x: torch.Tensor, act_buf: torch.Tensor,
                            ws: torch.Tensor, stream=None) -> torch.Tensor:
    L, I = x.shape
    _dev_f32(x, (L, I), "x")
    st = lib().hot_compress_activation(C.byref(cfg.c()), _ptr(x), L, I, _ptr(act_buf), _ptr(ws),
                                       ws.numel(), _stream(stream))
    _check(st, "hot_compress_activation")
    return act_buf


def hot_linear_backward_gx(cfg: Config, g_y: torch.Tensor, w: torch.Tensor, gy_quantizer: int,
                           g_x: torch.Tensor, ws: torch.Tensor, stream=None) -> torch.Tensor:
    L, O = g_y.shape
    I = w.shape[1]
    _dev_f32(g_y, (L, O), "g_y"); _dev_f32(w, (O, I), "w"); _dev_f32(g_x, (L, I), "g_x")
    st = lib().hot_linear_backward_gx(C.byref(cfg.c()), _ptr(g_y), _ptr(w), L, O, I,
                                      int(gy_quantizer), _ptr(g_x), _ptr(ws), ws.numel(),
                                      _stream(stream))
    _check(st, "hot_linear_backward_gx")
    return g_x


def hot_linear_backward_gx_noalloc(cfg: Config, g_y: torch.Tensor, w: torch.Tensor, gy_quantizer: int,
                                   g_x: torch.Tensor, stream=None) -> torch.Tensor:
    """hot_linear_backward_gx with the library's built-in scratch instead of a workspace."""
    L, O = g_y.shape
    I = w.shape[1]
    _dev_f32(g_y, (L, O), "g_y"); _dev_f32(w, (O, I), "w"); _dev_f32(g_x, (L, I), "g_x")
    st = lib().hot_linear_backward_gx_noalloc(C.byref(cfg.c()), _ptr(g_y), _ptr(w), L, O, I,
                                              int(gy_quantizer), _ptr(g_x), _stream(stream))
    _check(st, "hot_linear_backward_gx_noalloc")
    return g_x


def hot_linear_backward_gw(cfg: Config, g_y: torch.Tensor, act_buf: torch.Tensor, I: int,
                           g_w: torch.Tensor, ws: torch.Tensor, stream=None) -> torch.Tensor:
    L, O = g_y.shape
    _dev_f32(g_y, (L, O), "g_y"); _dev_f32(g_w, (O, I), "g_w")
    st = lib().hot_linear_backward_gw(C.byref(cfg.c()), _ptr(g_y), _ptr(act_buf), L, O, I,
                                      _ptr(g_w), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "hot_linear_backward_gw")
    return g_w


def hot_linear_backward(cfg: Config, g_y: torch.Tensor, w: torch.Tensor, act_buf: torch.Tensor,
                        gy_quantizer: int, g_x: torch.Tensor, g_w: torch.Tensor, ws: torch.Tensor,
                        stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    L, O = g_y.shape
    I = w.shape[1]
    _dev_f32(g_y, (L, O), "g_y"); _dev_f32(w, (O, I), "w")
    _dev_f32(g_x, (L, I), "g_x"); _dev_f32(g_w, (O, I), "g_w")
    st = lib().hot_linear_backward(C.byref(cfg.c()), _ptr(g_y), _ptr(w), _ptr(act_buf), L, O, I,
                                   int(gy_quantizer), _ptr(g_x), _ptr(g_w), _ptr(ws), ws.numel(),
                                   _stream(stream))
    _check(st, "hot_linear_backward")
    return g_x, g_w


def hot_select_quantizer(cfg: Config, g_y: torch.Tensor, ws: torch.Tensor,
                         stream=None) -> Tuple[int, float, float]:
    """Returns (choice, mse_token, mse_tensor)."""
    L, O = g_y.shape
    _dev_f32(g_y, (L, O), "g_y")
    choice, mt, mn = C.c_int(-1), C.c_double(0), C.c_double(0)
    st = lib().hot_select_quantizer(C.byref(cfg.c()), _ptr(g_y), L, O, C.byref(choice),
                                    C.byref(mt), C.byref(mn), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "hot_select_quantizer")
    return choice.value, mt.value, mn.value


def hot_lowpass_l1_rows(block: int, keep: int):
    """The `keep` low-pass rows of a block by the LP_L1 criterion, as a list for Config.keep_idx."""
    out = (C.c_int32 * keep)()
    _check(lib().hot_lowpass_l1_rows(int(block), int(keep), out), "hot_lowpass_l1_rows")
    return [int(k) for k in out]


def hot_debug_unpack_activation(cfg: Config, act_buf: torch.Tensor, L: int, I: int, stream=None):
    """Returns (codes int8 [L*r/n, I], scale float32 [1]) on the device; with gw_bits = 16
    the codes are bfloat16 bit patterns (int16) and the scale is 1."""
    Lr = cfg.reduced_tokens(L)
    codes = torch.empty((Lr, I), dtype=torch.int16 if cfg.gw_bits == 16 else torch.int8,
                        device=act_buf.device)
    scale = torch.empty(1, dtype=torch.float32, device=act_buf.device)
    st = lib().hot_debug_unpack_activation(C.byref(cfg.c()), _ptr(act_buf), L, I, _ptr(codes),
                                           _ptr(scale), _stream(stream))
    _check(st, "hot_debug_unpack_activation")
    return codes, scale


def hot_debug_gx_operands(cfg: Config, ws: torch.Tensor, L: int, O: int, I: int, gy_quantizer: int,
                          want_acc: bool = True, stream=None):
    """Returns dict(qg [L,O] int8, sg [L]|[1], qw [O,I] int8, sw [1], acc [L,I] int32)."""
    dev = ws.device
    qg = torch.empty((L, O), dtype=torch.int8, device=dev)
    sg = torch.empty(L if gy_quantizer == HOT_Q_PER_TOKEN else 1, dtype=torch.float32, device=dev)
    qw = torch.empty((O, I), dtype=torch.int8, device=dev)
    sw = torch.empty(1, dtype=torch.float32, device=dev)
    acc = torch.empty((L, I), dtype=torch.int32, device=dev) if want_acc else None
    st = lib().hot_debug_gx_operands(C.byref(cfg.c()), _ptr(ws), L, O, I, int(gy_quantizer),
                                     _ptr(qg), _ptr(sg), _ptr(qw), _ptr(sw), _ptr(acc),
                                     _stream(stream))
    _check(st, "hot_debug_gx_operands")
    return dict(qg=qg, sg=sg, qw=qw, sw=sw, acc=acc)


def hot_debug_gw_operands(cfg: Config, ws: torch.Tensor, act_buf: torch.Tensor, L: int, O: int,
                          I: int, want_acc: bool = True, stream=None):
    """Returns dict(qg [L*r/n,O] int8, sg [1], acc [O,I] int32); with gw_bits = 16 qg holds
    bfloat16 bit patterns (int16) and acc the fp32 accumulators (float32)."""
    dev = ws.device
    Lr = cfg.reduced_tokens(L)
    qg = torch.empty((Lr, O), dtype=torch.int16 if cfg.gw_bits == 16 else torch.int8, device=dev)
    sg = torch.empty(1, dtype=torch.float32, device=dev)
    acc = torch.empty((O, I), dtype=torch.int32, device=dev) if want_acc else None
    st = lib().hot_debug_gw_operands(C.byref(cfg.c()), _ptr(ws), _ptr(act_buf), L, O, I, _ptr(qg),
                                     _ptr(sg), _ptr(acc), _stream(stream))
    _check(st, "hot_debug_gw_operands")
    if acc is not None and cfg.gw_bits == 16:
        acc = acc.view(torch.float32)
    return dict(qg=qg, sg=sg, acc=acc)


def hot_debug_fused_operands(cfg: Config, ws: torch.Tensor, act_buf: torch.Tensor, L: int, O: int,
                             I: int, gy_quantizer: int, want_acc: bool = True, stream=None):
    """Operands of the last hot_linear_backward: dict(qg, sg, qw, sw, acc_gx, qgh, sgh, acc_gw)."""
    dev = ws.device
    Lr = cfg.reduced_tokens(L)
    qg = torch.empty((L, O), dtype=torch.int8, device=dev)
    sg = torch.empty(L if gy_quantizer == HOT_Q_PER_TOKEN else 1, dtype=torch.float32, device=dev)
    qw = torch.empty((O, I), dtype=torch.int8, device=dev)
    sw = torch.empty(1, dtype=torch.float32, device=dev)
    qgh = torch.empty((Lr, O), dtype=torch.int8, device=dev)
    sgh = torch.empty(1, dtype=torch.float32, device=dev)
    acc_gx = torch.empty((L, I), dtype=torch.int32, device=dev) if want_acc else None
    acc_gw = torch.empty((O, I), dtype=torch.int32, device=dev) if want_acc else None
    st = lib().hot_debug_fused_operands(C.byref(cfg.c()), _ptr(ws), _ptr(act_buf), L, O, I,
                                        int(gy_quantizer), _ptr(qg), _ptr(sg), _ptr(qw), _ptr(sw),
                                        _ptr(acc_gx), _ptr(qgh), _ptr(sgh), _ptr(acc_gw),
                                        _stream(stream))
    _check(st, "hot_debug_fused_operands")
    return dict(qg=qg, sg=sg, qw=qw, sw=sw, acc_gx=acc_gx, qgh=qgh, sgh=sgh, acc_gw=acc_gw)


def hot_debug_set_backward_strategy(strategy: int) -> None:
    """0 = library's choice, 1 = separate paths, 2 = shared g_y passes where they exist."""
    _check(lib().hot_debug_set_backward_strategy(int(strategy)), "hot_debug_set_backward_strategy")


def hot_debug_set_gemm_mode(mode: int) -> None:
    """0: library's choice, 1: one workgroup per output tile, s >= 2: s K slices where a split applies."""
    _check(lib().hot_debug_set_gemm_mode(int(mode)), "hot_debug_set_gemm_mode")


def hot_debug_set_exchange_wait_us(us: int) -> None:
    _check(lib().hot_debug_set_exchange_wait_us(int(us)), "hot_debug_set_exchange_wait_us")


def hot_debug_profile_begin() -> None:
    _check(lib().hot_debug_profile_begin(), "hot_debug_profile_begin")


def hot_debug_profile_end():
    """Returns {stage name: (total ms, launches)} for the stages that ran."""
    ms = (C.c_float * HOT_NUM_STAGES)()
    cnt = (C.c_int64 * HOT_NUM_STAGES)()
    _check(lib().hot_debug_profile_end(ms, cnt), "hot_debug_profile_end")
    return {lib().hot_debug_stage_name(i).decode(): (float(ms[i]), int(cnt[i]))
            for i in range(HOT_NUM_STAGES) if cnt[i]}


def hot_debug_profile_sequence():
    """Stage names of the recording closed by the last hot_debug_profile_end, in launch order."""
    n = int(lib().hot_debug_profile_sequence(None, 0))
    buf = (C.c_int32 * max(n, 1))()
    lib().hot_debug_profile_sequence(buf, n)
    return [lib().hot_debug_stage_name(int(buf[i])).decode() for i in range(n)]


def hot_debug_probe(kind: int, buf: torch.Tensor, iters: int = 1, stream=None) -> None:
    _check(lib().hot_debug_probe(int(kind), _ptr(buf), buf.numel() * buf.element_size(), int(iters),
                                 _stream(stream)), "hot_debug_probe")
