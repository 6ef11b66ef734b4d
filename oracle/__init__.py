"""CPU oracle for the HOT linear-backward path.  TEST INFRASTRUCTURE ONLY.

numpy-in / numpy-out wrappers around ``hot_oracle.c`` (built by ``build()`` with
gcc, no fast-math, no contraction).  Nothing under the product package imports
this; only the tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hot_oracle.c")
_LIB = os.path.join(_HERE, "libhot_oracle.so")

NEAREST_EVEN = 0
PSEUDO_STOCHASTIC = 1

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  IEEE fp32 semantics are kept: no fast-math,
    no FMA contraction, baseline x86-64 (SSE2) code generation."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_LIB)
        _lib.hot_oracle_select_quantizer.restype = C.c_int
        _lib.hot_oracle_sequency.restype = C.c_int
        _lib.hot_oracle_threads.restype = C.c_int
        for f in ("hot_oracle_igemm_nn", "hot_oracle_igemm_tn", "hot_oracle_backward_gx",
                  "hot_oracle_backward_gw"):
            getattr(_lib, f).restype = C.c_int64
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int8)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


i64 = C.c_int64


def threads() -> int:
    return int(lib().hot_oracle_threads())


def hadamard(n: int) -> np.ndarray:
    H = np.zeros((n, n), dtype=np.int8)
    lib().hot_oracle_hadamard(C.c_int(n), _p(H))
    return H


def fwht(v) -> np.ndarray:
    out = _f32(v).copy()
    lib().hot_oracle_fwht(_p(out), C.c_int(out.shape[0]))
    return out


def sequency(n: int, k: int) -> int:
    return int(lib().hot_oracle_sequency(C.c_int(n), C.c_int(k)))


def lowpass_index(n: int, r: int) -> np.ndarray:
    idx = np.zeros(r, dtype=np.int32)
    lib().hot_oracle_lowpass_index(C.c_int(n), C.c_int(r), _p(idx))
    return idx


def lowpass_l1_index(n: int, r: int) -> np.ndarray:
    """The r low-pass rows by the 2-D (LP_L1) criterion of Supp. B, as read in hot_oracle.c."""
    idx = np.zeros(r, dtype=np.int32)
    lib().hot_oracle_lowpass_l1_index(C.c_int(n), C.c_int(r), _p(idx))
    return idx


def transform_rows(g, n: int) -> np.ndarray:
    g = _f32(g)
    T = np.empty_like(g)
    lib().hot_oracle_transform_rows(_p(g), i64(g.shape[0]), i64(g.shape[1]), C.c_int(n), _p(T))
    return T


def hla(x, n: int, r: int, keep: Sequence[int]) -> np.ndarray:
    x = _f32(x)
    R, Cc = x.shape
    keep = _i32(keep)
    out = np.empty((R // n * r, Cc), dtype=np.float32)
    lib().hot_oracle_hla(_p(x), i64(R), i64(Cc), C.c_int(n), C.c_int(r), _p(keep), _p(out))
    return out


def quantize(t, bits: int, per_token: bool, rounding: int):
    t = _f32(t)
    rows, cols = t.shape
    codes = np.empty((rows, cols), dtype=np.int8)
    scales = np.empty(rows if per_token else 1, dtype=np.float32)
    lib().hot_oracle_quantize(_p(t), i64(rows), i64(cols), C.c_int(bits), C.c_int(int(per_token)),
                              C.c_int(rounding), _p(codes), _p(scales))
    return codes, scales


def igemm_nn(A, B):
    A, B = _i8(A), _i8(B)
    M, K = A.shape
    N = B.shape[1]
    acc = np.empty((M, N), dtype=np.int64)
    bad = lib().hot_oracle_igemm_nn(_p(A), _p(B), i64(M), i64(N), i64(K), _p(acc))
    return acc, int(bad)


def igemm_tn(A, B):
    A, B = _i8(A), _i8(B)
    K, M = A.shape
    N = B.shape[1]
    acc = np.empty((M, N), dtype=np.int64)
    bad = lib().hot_oracle_igemm_tn(_p(A), _p(B), i64(M), i64(N), i64(K), _p(acc))
    return acc, int(bad)


def dequant(acc, s_row, s_col: float, n: int) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    s_row = _f32(s_row).reshape(-1)
    M, N = acc.shape
    out = np.empty((M, N), dtype=np.float64)
    lib().hot_oracle_dequant(_p(acc), i64(M), i64(N), _p(s_row),
                             C.c_int(1 if s_row.shape[0] == M and M > 1 else 0),
                             C.c_float(float(s_col)), C.c_int(n), _p(out))
    return out


def backward_gx(g_y, w, n: int, bits: int = 4, per_token: bool = True,
                rounding: int = PSEUDO_STOCHASTIC, taps: bool = True):
    """Returns dict(g_x, qg, sg, qw, sw, acc, overflow)."""
    g_y, w = _f32(g_y), _f32(w)
    L, O = g_y.shape
    I = w.shape[1]
    g_x = np.empty((L, I), dtype=np.float64)
    qg = np.empty((L, O), dtype=np.int8) if taps else None
    sg = np.empty(L if per_token else 1, dtype=np.float32)
    qw = np.empty((O, I), dtype=np.int8) if taps else None
    sw = np.empty(1, dtype=np.float32)
    acc = np.empty((L, I), dtype=np.int64) if taps else None
    bad = lib().hot_oracle_backward_gx(_p(g_y), _p(w), i64(L), i64(O), i64(I), C.c_int(n),
                                       C.c_int(bits), C.c_int(int(per_token)), C.c_int(rounding),
                                       _p(g_x), _p(qg), _p(sg), _p(qw), _p(sw), _p(acc))
    return dict(g_x=g_x, qg=qg, sg=sg, qw=qw, sw=sw, acc=acc, overflow=int(bad))


def compress_activation(x, n: int, r: int, keep=None, bits: int = 8,
                        rounding: int = PSEUDO_STOCHASTIC):
    """Returns (codes [L*r/n, I] int8, scale float32)."""
    x = _f32(x)
    L, I = x.shape
    keep = lowpass_index(n, r) if keep is None else _i32(keep)
    codes = np.empty((L // n * r, I), dtype=np.int8)
    scale = np.empty(1, dtype=np.float32)
    lib().hot_oracle_compress_activation(_p(x), i64(L), i64(I), C.c_int(n), C.c_int(r), _p(keep),
                                         C.c_int(bits), C.c_int(rounding), _p(codes), _p(scale))
    return codes, scale[0]


def backward_gw(g_y, x_codes, x_scale, n: int, r: int, keep=None, bits: int = 8,
                rounding: int = PSEUDO_STOCHASTIC, taps: bool = True):
    """Returns dict(g_w, qg, sg, acc, overflow)."""
    g_y, x_codes = _f32(g_y), _i8(x_codes)
    L, O = g_y.shape
    I = x_codes.shape[1]
    Lr = L // n * r
    assert x_codes.shape[0] == Lr
    keep = lowpass_index(n, r) if keep is None else _i32(keep)
    g_w = np.empty((O, I), dtype=np.float64)
    qg = np.empty((Lr, O), dtype=np.int8) if taps else None
    sg = np.empty(1, dtype=np.float32)
    acc = np.empty((O, I), dtype=np.int64) if taps else None
    bad = lib().hot_oracle_backward_gw(_p(g_y), _p(x_codes), C.c_float(float(x_scale)), i64(L),
                                       i64(O), i64(I), C.c_int(n), C.c_int(r), _p(keep),
                                       C.c_int(bits), C.c_int(rounding), _p(g_w), _p(qg), _p(sg),
                                       _p(acc))
    return dict(g_w=g_w, qg=qg, sg=sg[0], acc=acc, overflow=int(bad))


def select_quantizer(g_y, n: int, bits: int = 4, rounding: int = PSEUDO_STOCHASTIC,
                     threshold: float = 0.5):
    """Returns (per_token: bool, mse_token, mse_tensor)."""
    g_y = _f32(g_y)
    L, O = g_y.shape
    mt, mn = C.c_double(0), C.c_double(0)
    ch = lib().hot_oracle_select_quantizer(_p(g_y), i64(L), i64(O), C.c_int(n), C.c_int(bits),
                                           C.c_int(rounding), C.c_double(threshold),
                                           C.byref(mt), C.byref(mn))
    return bool(ch), mt.value, mn.value


def exact_backward(g_y, x, w, want_gx: bool = True, want_gw: bool = True):
    g_y, x, w = _f32(g_y), _f32(x), _f32(w)
    L, O = g_y.shape
    I = w.shape[1]
    g_x = np.empty((L, I), dtype=np.float64) if want_gx else None
    g_w = np.empty((O, I), dtype=np.float64) if want_gw else None
    lib().hot_oracle_exact_backward(_p(g_y), _p(x), _p(w), i64(L), i64(O), i64(I), _p(g_x), _p(g_w))
    return g_x, g_w


# ---- bf16 variant of the weight-gradient path (Sec. 4.2 finds g_w the path that is
# sensitive to quantisation; the low-rank projection is kept, the integer quantiser is
# replaced by bfloat16 operands with a wide accumulator) ---------------------------------

def bf16_bits(a) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even.
    bfloat16 is the upper half of the fp32 pattern: add half an ulp of the kept part,
    plus its last bit for the tie rule, and truncate.  Inputs must be finite."""
    u = _f32(a).view(np.uint32).astype(np.uint64)
    kept_lsb = (u >> 16) & 1
    return ((u + 0x7FFF + kept_lsb) >> 16).astype(np.uint16)


def bf16_value(bits) -> np.ndarray:
    """bfloat16 bit patterns -> the fp32 values they denote."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def compress_activation_bf16(x, n: int, r: int, keep=None) -> np.ndarray:
    """HLA(x) along the tokens (same transform as compress_activation), stored as bfloat16:
    returns the bit patterns [L*r/n, I] (uint16)."""
    keep = lowpass_index(n, r) if keep is None else _i32(keep)
    return bf16_bits(hla(x, n, r, keep))


def backward_gw_bf16(g_y, x_bits, n: int, r: int, keep=None):
    """g_w = HLA(g_y)^T . x_hat / n with both operands rounded to bfloat16 and the sum in
    double (a product of two bfloat16 values is exact in double).
    Returns dict(g_w [O, I] float64, gh_bits [L*r/n, O] uint16)."""
    keep = lowpass_index(n, r) if keep is None else _i32(keep)
    gh_bits = bf16_bits(hla(g_y, n, r, keep))
    A = bf16_value(gh_bits).astype(np.float64)
    B = bf16_value(x_bits).astype(np.float64)
    return dict(g_w=(A.T @ B) / float(n), gh_bits=gh_bits)


# ---- per-sample tiling of the token axis (the paper's ViT sequences have 197 tokens, not a
# multiple of the block size, and it does not say how they are tiled) ---------------------

def pad_samples(a, sample_tokens: int, n: int) -> np.ndarray:
    """[B*S, C] -> [B*S', C] with S' = S rounded up to a multiple of n: every sample of S
    tokens is followed by S' - S zero tokens, so that consecutive blocks of n never straddle
    two samples.  Every token-direction function above applied to the padded tensors is the
    per-sample definition (zero tokens add nothing to g_w)."""
    a = _f32(a)
    S = int(sample_tokens)
    assert S > 0 and a.shape[0] % S == 0
    B, Sp = a.shape[0] // S, -(-S // n) * n
    out = np.zeros((B, Sp, a.shape[1]), dtype=np.float32)
    out[:, :S, :] = a.reshape(B, S, a.shape[1])
    return out.reshape(B * Sp, a.shape[1])
