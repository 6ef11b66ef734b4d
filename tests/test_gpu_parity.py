"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element on the same seeded inputs.  Integer stages - codes, scales (fp32 bit
patterns) and int32 accumulators - must be identical; dequantised fp32 outputs
must agree within 1e-5 relative in max-norm (fp32 epilogue: one int->float
conversion and two multiplies, ~2e-7)."""
import sys

import numpy as np
import pytest
import torch

import hot_inputs
import oracle

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5


def _hot():
    import paper_2503_21261_amd as hot
    return hot


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def assert_close_maxnorm(got, ref, what, exact_accumulators=True):
    """The stated bound, 1e-5 of max|ref| on every element, and, where the accumulators are
    exact integers, an element-wise one that also holds small entries to their own size:
    |got - ref| <= 1e-5 |ref| + 1e-6 max|ref| (the epilogue's own error is about 2e-7 relative:
    one int->float conversion, two multiplies).  The bfloat16 variant sums its products in fp32
    on the matrix cores: an entry that is a small sum of K large cancelling terms (outlier
    tokens) carries an error of up to K 2^-24 of the terms' magnitude, not of its own, so only
    the stated max-norm bound applies there."""
    denom = np.max(np.abs(ref))
    diff = np.abs(got.astype(np.float64) - ref)
    err = np.max(diff)
    assert err <= REL_TOL * denom + 1e-300, f"{what}: max err {err:.3e} vs max|ref| {denom:.3e}"
    if not exact_accumulators:
        return
    excess = diff - (REL_TOL * np.abs(ref) + 1e-6 * denom)
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, (f"{what}: element {worst}: got {got[worst]!r}, ref {ref[worst]!r}, "
                                f"max|ref| {denom:.3e}")


def dequant_fp32(acc, s_row, s_col, n):
    """The epilogue's own arithmetic, in fp32 in its order: float(acc) * (s_row * (s_col / n));
    1/n is a power of two, so every step is one IEEE operation (the INT4 kernels carry 256 x acc
    and fold 1/256 into the factor: exact scalings that change no rounding)."""
    cs = np.float32(s_col) * np.float32(1.0 / n)
    rs = np.asarray(s_row, np.float32).reshape(-1, 1) * cs
    return np.asarray(acc).astype(np.float32) * rs


def assert_output_is_dequantised_accumulator(out, acc, s_row, s_col, n, what):
    """Ties the output of a production launch (fused epilogue, split-K hand-over) to the
    integer accumulators, which are compared exactly with the oracle: same bits everywhere.
    `out`, `acc`: device tensors; s_row: device [M] or [1]; s_col: device [1]."""
    cs = s_col.to(torch.float32) * torch.tensor(1.0 / n, dtype=torch.float32, device=out.device)
    rs = s_row.to(torch.float32).reshape(-1, 1) * cs
    assert torch.equal(out, acc.to(torch.float32) * rs), f"{what}: output is not float(acc) * scales"


def bits_equal(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


def check_gx(hot, cfg, gy, w, per_token, what):
    L, O = gy.shape
    I = w.shape[1]
    _say(f"[gx] {what} L={L} O={O} I={I} n={cfg.block} bits={cfg.gx_bits} token={per_token} round={cfg.rounding}")
    ref = oracle.backward_gx(gy.numpy(), w.numpy(), cfg.block, bits=cfg.gx_bits, per_token=per_token,
                             rounding=cfg.rounding)
    assert ref["overflow"] == 0
    gyd, wd = gy.cuda(), w.cuda()
    ws = hot.alloc_workspace(cfg, L, O, I)
    gx = torch.empty((L, I), dtype=torch.float32, device="cuda")
    q = hot.HOT_Q_PER_TOKEN if per_token else hot.HOT_Q_PER_TENSOR
    hot.hot_linear_backward_gx(cfg, gyd, wd, q, gx, ws)
    taps = hot.hot_debug_gx_operands(cfg, ws, L, O, I, q)
    torch.cuda.synchronize()
    assert bits_equal(taps["sg"].cpu().numpy(), ref["sg"]), f"{what}: g_y scales differ"
    assert bits_equal(taps["sw"].cpu().numpy(), ref["sw"]), f"{what}: w scale differs"
    assert np.array_equal(taps["qg"].cpu().numpy(), ref["qg"]), f"{what}: g_y codes differ"
    assert np.array_equal(taps["qw"].cpu().numpy(), ref["qw"]), f"{what}: w codes differ"
    assert np.array_equal(taps["acc"].cpu().numpy().astype(np.int64), ref["acc"]), f"{what}: accumulators differ"
    assert_close_maxnorm(gx.cpu().numpy(), ref["g_x"], what + " g_x")
    assert_output_is_dequantised_accumulator(gx, taps["acc"], taps["sg"], taps["sw"], cfg.block, what + " g_x")
    assert np.array_equal(gx.cpu().numpy(), dequant_fp32(ref["acc"], ref["sg"], ref["sw"][0], cfg.block)), \
        f"{what}: g_x is not the fp32 dequantisation of the oracle's accumulators"
    return ref, gx


def check_gw(hot, cfg, gy, x, what):
    L, O = gy.shape
    I = x.shape[1]
    _say(f"[gw] {what} L={L} O={O} I={I} n={cfg.block} r={cfg.keep} keep={cfg.keep_idx} round={cfg.rounding}")
    keep = None if cfg.keep_idx is None else list(cfg.keep_idx)
    S = cfg.sample_tokens
    xo = oracle.pad_samples(x.numpy(), S, cfg.block) if S else x.numpy()
    gyo = oracle.pad_samples(gy.numpy(), S, cfg.block) if S else gy.numpy()
    codes_ref, sx_ref = oracle.compress_activation(xo, cfg.block, cfg.keep, keep=keep,
                                                   rounding=cfg.rounding)
    ref = oracle.backward_gw(gyo, codes_ref, sx_ref, cfg.block, cfg.keep, keep=keep,
                             rounding=cfg.rounding)
    assert ref["overflow"] == 0
    gyd, xd = gy.cuda(), x.cuda()
    act = hot.alloc_act_buffer(cfg, L, I)
    ws = hot.alloc_workspace(cfg, L, O, I)
    hot.hot_compress_activation(cfg, xd, act, ws)
    codes, sx = hot.hot_debug_unpack_activation(cfg, act, L, I)
    gw = torch.empty((O, I), dtype=torch.float32, device="cuda")
    hot.hot_linear_backward_gw(cfg, gyd, act, I, gw, ws)
    taps = hot.hot_debug_gw_operands(cfg, ws, act, L, O, I)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), [sx_ref]), f"{what}: activation scale differs"
    assert np.array_equal(codes.cpu().numpy(), codes_ref), f"{what}: activation codes differ"
    assert bits_equal(taps["sg"].cpu().numpy(), [ref["sg"]]), f"{what}: HLA(g_y) scale differs"
    assert np.array_equal(taps["qg"].cpu().numpy(), ref["qg"]), f"{what}: HLA(g_y) codes differ"
    assert np.array_equal(taps["acc"].cpu().numpy().astype(np.int64), ref["acc"]), f"{what}: accumulators differ"
    assert_close_maxnorm(gw.cpu().numpy(), ref["g_w"], what + " g_w")
    assert_output_is_dequantised_accumulator(gw, taps["acc"], taps["sg"], sx, cfg.block, what + " g_w")
    assert np.array_equal(gw.cpu().numpy(), dequant_fp32(ref["acc"], [ref["sg"]], sx_ref, cfg.block)), \
        f"{what}: g_w is not the fp32 dequantisation of the oracle's accumulators"
    return ref, gw


def make(L, O, I, seed, gy_kind="chan_outlier", x_kind="normal"):
    name = f"t{L}x{O}x{I}"
    return (hot_inputs.make_x(x_kind, L, I, seed, name), hot_inputs.make_w(O, I, seed, name),
            hot_inputs.make_gy(gy_kind, L, O, seed, name))


# shapes span several 128x128 GEMM tiles, ragged M/N tails, K that is / is not a
# multiple of the 128-byte operand pitch, and rows that fill 1..many register slots
GX_SHAPES = [
    (16, 16, 4),        # one block, one tile
    (1, 64, 1),         # single token, single input channel
    (48, 64, 40),
    (130, 160, 72),     # ragged everywhere
    (257, 1040, 130),   # row longer than one wave's 4 slots (workgroup-per-row variant)
    (300, 2304, 200),
]


@pytest.mark.parametrize("n", [16, 32, 64])
@pytest.mark.parametrize("shape", GX_SHAPES)
def test_gx_small_shapes_per_token(n, shape):
    L, O, I = shape
    if O % n:
        pytest.skip("O not a multiple of n")
    hot = _hot()
    x, w, gy = make(L, O, I, seed=3)
    check_gx(hot, hot.Config(block=n, keep=n // 2), gy, w, True, "small")


@pytest.mark.parametrize("n,bits,rounding", [(16, 4, 0), (16, 8, 1), (32, 8, 0), (64, 4, 1)])
@pytest.mark.parametrize("per_token", [True, False])
def test_gx_variants(n, bits, rounding, per_token):
    hot = _hot()
    x, w, gy = make(200, 384, 136, seed=5, gy_kind="tok_outlier")
    cfg = hot.Config(block=n, keep=n // 2, gx_bits=bits, rounding=rounding)
    check_gx(hot, cfg, gy, w, per_token, "variant")


def test_gx_config1_full():
    """configs[0]: L=512, O=768, I=768, n=16, INT4 per token."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg1_single_512x768x768"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    ref, gx = check_gx(hot, cfg, gy, w, True, "cfg1")
    check_gx(hot, cfg, gy, w, False, "cfg1 per-tensor")
    exact, _ = oracle.exact_backward(gy.numpy(), x.numpy(), w.numpy(), want_gw=False)
    rel = np.linalg.norm(gx.cpu().numpy() - exact) / np.linalg.norm(exact)
    _say(f"cfg1 g_x relative Frobenius error vs exact backward (statistic): {rel:.4f}")


def test_gx_long_rows_register_limit_and_streaming():
    hot = _hot()
    for O in (16384, 16448):   # largest register-resident row; first streamed row
        x, w, gy = make(5, O, 24, seed=7, gy_kind="t4")
        check_gx(hot, hot.Config(block=64, keep=32), gy, w, True, f"long row O={O}")
        check_gx(hot, hot.Config(block=16, keep=8), gy, w, False, f"long row O={O}")


def test_gx_zero_inputs_give_zero():
    hot = _hot()
    cfg = hot.Config()
    gy = torch.zeros(64, 64)
    w = hot_inputs.make_w(64, 32, 0, "z")
    gy[3] = hot_inputs.normal((64,), 1e-3, 0, "zrow")  # one live token among zero tokens
    ref, gx = check_gx(hot, cfg, gy, w, True, "zero rows")
    assert not gx.cpu().numpy()[0].any()
    ref, gx = check_gx(hot, cfg, torch.zeros(64, 64), w, False, "all zero")
    assert not gx.cpu().numpy().any()


GW_CASES = [
    # L, O, I, n, r, keep_idx
    (16, 8, 4, 16, 8, None),
    (64, 40, 24, 16, 8, None),
    (272, 130, 72, 16, 8, None),     # L' = 136: not a multiple of the operand pitch
    (512, 200, 136, 32, 16, None),
    (1024, 96, 260, 64, 32, None),
    (256, 64, 64, 16, 16, None),     # full rank
    (256, 64, 64, 16, 1, None),      # rank 1: block means
    (240, 64, 72, 16, 3, None),      # odd rank
    (256, 64, 64, 16, 4, [5, 0, 9, 14]),   # caller-supplied rows
    (2048, 300, 140, 16, 8, None),   # several K stages and split-K slices
]


@pytest.mark.parametrize("case", GW_CASES)
def test_gw_small_shapes(case):
    L, O, I, n, r, keep = case
    hot = _hot()
    x, w, gy = make(L, O, I, seed=11, gy_kind="t4")
    check_gw(hot, hot.Config(block=n, keep=r, keep_idx=keep), gy, x, "small")


@pytest.mark.parametrize("n,r,shape", [(16, 8, (512, 200, 136)), (16, 6, (272, 130, 72)), (64, 16, (1024, 96, 260)),
                                       (32, 16, (2048, 300, 140)), (16, 8, (50432, 768, 768))])
def test_gw_with_lp_l1_rows(n, r, shape):
    """The paper's own choice of kept rows (Supp. B: top r by the LP_L1 criterion) passed as
    keep_idx: activation compression and the g_w path on the generic kept-row kernels, INT8 and
    bfloat16, the last shape at config 3's full token count."""
    L, O, I = shape
    hot = _hot()
    keep = hot.hot_lowpass_l1_rows(n, r)
    assert keep == oracle.lowpass_l1_index(n, r).tolist()
    x, w, gy = make(L, O, I, seed=91, gy_kind="t4")
    check_gw(hot, hot.Config(block=n, keep=r, keep_idx=keep), gy, x, "LP_L1 rows")
    if L <= 4096:
        check_gw_bf16(hot, hot.Config(block=n, keep=r, keep_idx=keep, gw_bits=16), gy, x, "LP_L1 rows bf16")
        Oc = O // n * n
        check_fused(hot, hot.Config(block=n, keep=r, keep_idx=keep), gy[:, :Oc].contiguous(), x, w[:Oc].contiguous(),
                    True, "LP_L1 rows, one call")


def test_gw_nearest_even_and_bf16_inputs():
    hot = _hot()
    x, w, gy = make(512, 96, 80, seed=13, x_kind="bf16")
    check_gw(hot, hot.Config(block=32, keep=16, rounding=0), gy, x, "rne")


def test_gw_config1_full():
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg1_single_512x768x768"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    ref, gw = check_gw(hot, cfg, gy, x, "cfg1")
    L, I = x.shape
    assert hot.hot_act_buffer_bytes(cfg, L, I) == 256 + (4 * L * I) // 8  # 12.5 % of fp32 (Sec. 5.2.1)
    _, exact = oracle.exact_backward(gy.numpy(), x.numpy(), w.numpy(), want_gx=False)
    rel = np.linalg.norm(gw.cpu().numpy() - exact) / np.linalg.norm(exact)
    _say(f"cfg1 g_w relative Frobenius error vs exact backward (statistic): {rel:.4f}")


@pytest.mark.parametrize("kind,n", [("tok_outlier", 16), ("chan_outlier", 16), ("t3", 64), ("normal", 32)])
def test_select_quantizer_matches_oracle(kind, n):
    hot = _hot()
    L, O = 384, 512
    gy = hot_inputs.make_gy(kind, L, O, 17, "sel")
    _say(f"[select] kind={kind} n={n} L={L} O={O}")
    cfg = hot.Config(block=n, keep=n // 2)
    ws = hot.alloc_workspace(cfg, L, O, 64)
    choice, m_tok, m_ten = hot.hot_select_quantizer(cfg, gy.cuda(), ws)
    ref_choice, r_tok, r_ten = oracle.select_quantizer(gy.numpy(), n, bits=4, rounding=cfg.rounding,
                                                       threshold=cfg.lqs_threshold)
    # same codes and scales on both sides; only the order of the double sums differs
    np.testing.assert_allclose(m_tok, r_tok, rtol=1e-10)
    np.testing.assert_allclose(m_ten, r_ten, rtol=1e-10)
    assert choice == int(ref_choice)
    if kind == "tok_outlier":
        assert choice == hot.HOT_Q_PER_TOKEN
    if kind == "normal":
        assert choice == hot.HOT_Q_PER_TENSOR


def test_select_quantizer_zero_gradient():
    hot = _hot()
    cfg = hot.Config()
    ws = hot.alloc_workspace(cfg, 32, 64, 16)
    choice, m_tok, m_ten = hot.hot_select_quantizer(cfg, torch.zeros(32, 64, device="cuda"), ws)
    assert (choice, m_tok, m_ten) == (hot.HOT_Q_PER_TENSOR, 0.0, 0.0)


def test_calls_are_repeatable_and_stream_ordered():
    """Same inputs, same workspace, non-default stream: identical bits every time."""
    hot = _hot()
    x, w, gy = make(304, 320, 200, seed=19)
    cfg = hot.Config()
    L, O = gy.shape
    I = w.shape[1]
    gyd, wd, xd = gy.cuda(), w.cuda(), x.cuda()
    ws = hot.alloc_workspace(cfg, L, O, I)
    act = hot.alloc_act_buffer(cfg, L, I)
    outs = []
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(3):
        gx = torch.empty((L, I), device="cuda")
        gw = torch.empty((O, I), device="cuda")
        with torch.cuda.stream(s):
            hot.hot_compress_activation(cfg, xd, act, ws, stream=s)
            hot.hot_linear_backward_gx(cfg, gyd, wd, hot.HOT_Q_PER_TOKEN, gx, ws, stream=s)
            hot.hot_linear_backward_gw(cfg, gyd, act, I, gw, ws, stream=s)
        s.synchronize()
        outs.append((gx.cpu().numpy().copy(), gw.cpu().numpy().copy()))
    for gx, gw in outs[1:]:
        assert np.array_equal(gx, outs[0][0]) and np.array_equal(gw, outs[0][1])


# ---- full-size and workload-shaped cases -------------------------------------------------

def test_config2_full_size_in_bench_configuration():
    """configs[1] (ViT-B fc1, 12608 tokens, n=32, r=16) exactly as bench.py launches it;
    the oracle is fast enough to compare every element of every stage."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg2_vitb_fc1"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    check_gx(hot, cfg, gy, w, True, "cfg2 per-token")
    check_gx(hot, cfg, gy, w, False, "cfg2 per-tensor")
    check_gw(hot, cfg, gy, x, "cfg2")
    check_fused(hot, cfg, gy, x, w, True, "cfg2 one call, per-token")
    check_fused(hot, cfg, gy, x, w, False, "cfg2 one call, per-tensor")
    L, I = x.shape
    # 12.5 % of fp32 plus the row padding to 128 bytes and the header
    assert hot.hot_act_buffer_bytes(cfg, L, I) == 256 + I * ((L // 2 + 127) // 128 * 128)


@pytest.mark.parametrize("name,L", [("cfg3_vitb_block_b256", 1024), ("cfg4_llm7b_mlp", 256),
                                    ("cfg5_vitl_chain", 512)])
def test_workload_shaped_layers_on_a_token_subrange(name, L):
    """Layers of configs[2..4] at their real O, I, block and value distributions on a
    token sub-range the oracle finishes in seconds; config 4 takes its quantizer from
    hot_select_quantizer, which must agree with the oracle's choice."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS[name]
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    for layer in wl.layers:
        x, w, gy = hot_inputs.make_layer(wl, layer, seed=0, L=L)
        per_token = wl.quantizer == "token"
        if wl.quantizer == "select":
            ws = hot.alloc_workspace(cfg, L, layer.O, layer.I)
            choice, m_tok, m_ten = hot.hot_select_quantizer(cfg, gy.cuda(), ws)
            ref_choice, r_tok, r_ten = oracle.select_quantizer(gy.numpy(), wl.block)
            assert choice == int(ref_choice)
            np.testing.assert_allclose([m_tok, m_ten], [r_tok, r_ten], rtol=1e-10)
            per_token = bool(choice)
            _say(f"[select] {name}.{layer.name}: {'token' if per_token else 'tensor'} "
                 f"mse_token={m_tok:.3e} mse_tensor={m_ten:.3e}")
        check_gx(hot, cfg, gy, w, per_token, f"{name}.{layer.name}")
        check_gw(hot, cfg, gy, x, f"{name}.{layer.name}")
        check_fused(hot, cfg, gy, x, w, per_token, f"{name}.{layer.name}")


def _amax_of(A):
    return 127.0 if A.dtype == np.int8 else float(2 ** 31)


def _matvec_exact(A, v, chunk=16384):
    """A @ v for integer A (int8 codes or int32 accumulators) and integer v, exactly, in row
    chunks (no full-size wide copy of A): float64 BLAS when every sum stays below 2^53,
    else int64."""
    v = np.asarray(v)
    if float(np.abs(v.astype(np.float64)).sum()) * _amax_of(A) < 2.0 ** 53:
        vf = v.astype(np.float64)
        out = np.concatenate([A[i:i + chunk].astype(np.float64) @ vf for i in range(0, A.shape[0], chunk)])
        return np.rint(out).astype(np.int64)
    vi = v.astype(np.int64)
    return np.concatenate([A[i:i + chunk].astype(np.int64) @ vi for i in range(0, A.shape[0], chunk)])


def _vecmat_exact(u, A, chunk=16384):
    """u @ A, same rules, accumulated over row chunks of A."""
    u = np.asarray(u)
    if float(np.abs(u.astype(np.float64)).sum()) * _amax_of(A) < 2.0 ** 53:
        uf = u.astype(np.float64)
        out = np.zeros(A.shape[1], dtype=np.float64)
        for i in range(0, A.shape[0], chunk):
            out += uf[i:i + chunk] @ A[i:i + chunk].astype(np.float64)
        return np.rint(out).astype(np.int64)
    ui = u.astype(np.int64)
    out = np.zeros(A.shape[1], dtype=np.int64)
    for i in range(0, A.shape[0], chunk):
        out += ui[i:i + chunk] @ A[i:i + chunk].astype(np.int64)
    return out


class FullSizeRefs:
    """Oracle stages of one layer at its full size, computed once: every code and scale of the
    four quantised operands, and what the integer products must satisfy: the exact Freivalds
    images A (B v) and (u A) B for random small-integer vectors (checked on all outputs), and
    the oracle's own GEMM on sampled output rows, whose dequantised rows bound the fp32 outputs."""

    def __init__(self, x, w, gy, n, r, per_token, seed=5):
        self.n, self.r, self.per_token = n, r, per_token
        L, O = gy.shape
        I = w.shape[1]
        self.L, self.O, self.I = L, O, I
        rng = np.random.default_rng(seed)
        PSR = oracle.PSEUDO_STOCHASTIC
        self.qg, self.sg = oracle.quantize(oracle.transform_rows(gy, n), 4, per_token, PSR)
        self.qw, self.sw = oracle.quantize(oracle.hla(w, n, n, np.arange(n)), 4, False, PSR)
        keep = oracle.lowpass_index(n, r)
        self.xc, self.sx = oracle.compress_activation(x, n, r)
        self.gh, self.sh = oracle.quantize(oracle.hla(gy, n, r, keep), 8, False, PSR)
        # g_x product [L x I] = qg [L x O] . qw [O x I]
        self.vx = rng.integers(-2048, 2048, size=I)
        self.ux = rng.integers(-2048, 2048, size=L)
        self.gx_Cv = _matvec_exact(self.qg, _matvec_exact(self.qw, self.vx))
        self.gx_uC = _vecmat_exact(_vecmat_exact(self.ux, self.qg), self.qw)
        self.rows = np.unique(np.concatenate([np.arange(0, 256), rng.integers(0, L, 512), np.arange(L - 200, L)]))
        self.gx_acc_rows, bad = oracle.igemm_nn(self.qg[self.rows], self.qw)
        assert bad == 0
        self.gx_rows = oracle.dequant(self.gx_acc_rows, self.sg[self.rows] if per_token else self.sg, self.sw[0], n)
        # g_w product [O x I] = gh^T [O x L'] . xc [L' x I]
        self.vw = rng.integers(-2048, 2048, size=I)
        self.uw = rng.integers(-2048, 2048, size=O)
        self.gw_Cv = _vecmat_exact(_matvec_exact(self.xc, self.vw), self.gh)
        self.gw_uC = _vecmat_exact(_matvec_exact(self.gh, self.uw), self.xc)
        self.orow = np.unique(np.concatenate([np.arange(0, 64), rng.integers(0, O, 64), np.arange(O - 40, O)]))
        self.gw_acc_rows, bad = oracle.igemm_tn(np.ascontiguousarray(self.gh[:, self.orow]), self.xc)
        assert bad == 0
        self.gw_rows = oracle.dequant(self.gw_acc_rows, self.sh, self.sx, n)

    def check_gx_operands(self, qg, sg, qw, sw, what):
        assert np.array_equal(qg.cpu().numpy(), self.qg), f"{what}: g_y codes differ"
        assert bits_equal(sg.cpu().numpy(), self.sg), f"{what}: g_y scales differ"
        assert np.array_equal(qw.cpu().numpy(), self.qw), f"{what}: w codes differ"
        assert bits_equal(sw.cpu().numpy(), self.sw), f"{what}: w scale differs"

    def check_gx_product(self, acc_d, gx_d, sg_d, sw_d, what):
        acc = acc_d.cpu().numpy()
        assert np.array_equal(_matvec_exact(acc, self.vx), self.gx_Cv), f"{what}: g_x accumulators, C v"
        assert np.array_equal(_vecmat_exact(self.ux, acc), self.gx_uC), f"{what}: g_x accumulators, u C"
        assert np.array_equal(acc[self.rows].astype(np.int64), self.gx_acc_rows), f"{what}: g_x accumulator rows"
        del acc
        self.check_gx_output(gx_d, what)
        assert_output_is_dequantised_accumulator(gx_d, acc_d, sg_d, sw_d, self.n, what + " g_x")

    def check_gx_output(self, gx_d, what):
        got = gx_d[torch.from_numpy(self.rows).cuda()].cpu().numpy()
        assert_close_maxnorm(got, self.gx_rows, what + " g_x rows")
        want = dequant_fp32(self.gx_acc_rows, self.sg[self.rows] if self.per_token else self.sg, self.sw[0], self.n)
        assert np.array_equal(got, want), f"{what}: g_x rows are not the fp32 dequantisation of the oracle's sums"

    def check_gw_operands(self, codes, sx, qgh, sgh, what):
        if codes is not None:
            assert bits_equal(sx.cpu().numpy(), [self.sx]) and np.array_equal(codes.cpu().numpy(), self.xc), \
                f"{what}: compressed activation differs"
        assert bits_equal(sgh.cpu().numpy(), self.sh), f"{what}: HLA(g_y) scale differs"
        assert np.array_equal(qgh.cpu().numpy(), self.gh), f"{what}: HLA(g_y) codes differ"

    def check_gw_product(self, acc_d, gw_d, sgh_d, sx_d, what):
        acc = acc_d.cpu().numpy()
        assert np.array_equal(_matvec_exact(acc, self.vw), self.gw_Cv), f"{what}: g_w accumulators, C v"
        assert np.array_equal(_vecmat_exact(self.uw, acc), self.gw_uC), f"{what}: g_w accumulators, u C"
        assert np.array_equal(acc[self.orow].astype(np.int64), self.gw_acc_rows), f"{what}: g_w accumulator rows"
        self.check_gw_output(gw_d, what)
        assert_output_is_dequantised_accumulator(gw_d, acc_d, sgh_d, sx_d, self.n, what + " g_w")

    def check_gw_output(self, gw_d, what):
        got = gw_d.cpu().numpy()[self.orow]
        assert_close_maxnorm(got, self.gw_rows, what + " g_w rows")
        assert np.array_equal(got, dequant_fp32(self.gw_acc_rows, self.sh, self.sx, self.n)), \
            f"{what}: g_w rows are not the fp32 dequantisation of the oracle's sums"


def check_full_size_layer(hot, cfg, xd, wd, gyd, per_token, what, one_call_strategies=(0, 2)):
    """One layer at its full size through every way the library computes it: the two separate
    calls, then hot_linear_backward under each strategy given (0 = the library's own choice,
    which is what the benchmark's sweeps time; 2 = the shared g_y passes wherever they exist).
    Where the one-call form ran the shared passes, all its operands and both accumulators are
    compared with the oracle again; where it ran the separate paths its outputs must be the
    separate calls' bits.  Returns (g_x, g_w) of the default strategy."""
    L, O = gyd.shape
    I = wd.shape[1]
    n, r = cfg.block, cfg.keep
    _say(f"[full] {what} L={L} O={O} I={I} n={n} r={r} token={per_token}: oracle stages")
    refs = FullSizeRefs(xd.cpu().numpy(), wd.cpu().numpy(), gyd.cpu().numpy(), n, r, per_token)
    ws = hot.alloc_workspace(cfg, L, O, I)
    act = hot.alloc_act_buffer(cfg, L, I)
    q = hot.HOT_Q_PER_TOKEN if per_token else hot.HOT_Q_PER_TENSOR

    _say(f"[full] {what}: separate calls")
    gx = torch.empty((L, I), device="cuda")
    hot.hot_linear_backward_gx(cfg, gyd, wd, q, gx, ws)
    t = hot.hot_debug_gx_operands(cfg, ws, L, O, I, q)
    torch.cuda.synchronize()
    refs.check_gx_operands(t["qg"], t["sg"], t["qw"], t["sw"], what)
    refs.check_gx_product(t["acc"], gx, t["sg"], t["sw"], what)
    del t
    hot.hot_compress_activation(cfg, xd, act, ws)
    codes, sx = hot.hot_debug_unpack_activation(cfg, act, L, I)
    gw = torch.empty((O, I), device="cuda")
    hot.hot_linear_backward_gw(cfg, gyd, act, I, gw, ws)
    t = hot.hot_debug_gw_operands(cfg, ws, act, L, O, I)
    torch.cuda.synchronize()
    refs.check_gw_operands(codes, sx, t["qg"], t["sg"], what)
    refs.check_gw_product(t["acc"], gw, t["sg"], sx, what)
    del t, codes

    out = (gx, gw)
    for strategy in one_call_strategies:
        _say(f"[full] {what}: hot_linear_backward, strategy {strategy}")
        gx1 = torch.full((L, I), float("nan"), device="cuda")
        gw1 = torch.full((O, I), float("nan"), device="cuda")
        ws.fill_(0x5A)
        hot.hot_debug_set_backward_strategy(strategy)
        try:
            hot.hot_linear_backward(cfg, gyd, wd, act, q, gx1, gw1, ws)
            try:
                t = hot.hot_debug_fused_operands(cfg, ws, act, L, O, I, q)
            except hot.HotError as e:       # this strategy ran the separate paths for this shape
                assert e.status == hot.HOT_ERR_UNIMPLEMENTED
                t = None
        finally:
            hot.hot_debug_set_backward_strategy(0)
        torch.cuda.synchronize()
        assert torch.equal(gx1, gx) and torch.equal(gw1, gw), f"{what}: strategy {strategy} differs from the separate calls"
        if t is not None:
            _say(f"[full] {what}: strategy {strategy} ran the shared g_y passes")
            refs.check_gx_operands(t["qg"], t["sg"], t["qw"], t["sw"], what + " (shared passes)")
            refs.check_gx_product(t["acc_gx"], gx1, t["sg"], t["sw"], what + " (shared passes)")
            refs.check_gw_operands(None, None, t["qgh"], t["sgh"], what + " (shared passes)")
            refs.check_gw_product(t["acc_gw"], gw1, t["sgh"], sx, what + " (shared passes)")
        elif strategy == 0:
            assert n != 16 or refs.gh.size * 4 <= 80e6, f"{what}: expected the shared passes by default"
        if strategy == 0:
            out = (gx1, gw1)
        del t
    return out


@pytest.mark.parametrize("name,idx", [("cfg3_vitb_block_b256", 0), ("cfg3_vitb_block_b256", 1),
                                      ("cfg3_vitb_block_b256", 2), ("cfg3_vitb_block_b256", 3),
                                      ("cfg4_llm7b_mlp", 0), ("cfg4_llm7b_mlp", 1),
                                      ("cfg5_vitl_chain", 0), ("cfg5_vitl_chain", 1)])
def test_full_size_layers_sampled(name, idx):
    """Every layer of configs[2], [3] and [4] at its full token count (config 4: the 256x256
    GEMM tiles, 64-row blocks and the quantiser hot_select_quantizer picks at that size, which
    must be the oracle's; config 5: tensors beyond 2^31 bytes on either side), through the
    separate calls and through hot_linear_backward as the sweeps of the benchmark call it."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS[name]
    layer = wl.layers[idx]
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    xd, wd, gyd = hot_inputs.make_layer(wl, layer, seed=0, device="cuda")
    per_token = wl.quantizer == "token"
    if wl.quantizer == "select":
        ws = hot.alloc_workspace(cfg, layer.L, layer.O, layer.I)
        choice, m_tok, m_ten = hot.hot_select_quantizer(cfg, gyd, ws)
        ref_choice, r_tok, r_ten = oracle.select_quantizer(gyd.cpu().numpy(), wl.block)
        _say(f"[select] {name}.{layer.name} full size: {'token' if choice else 'tensor'} "
             f"mse_token={m_tok:.6e} mse_tensor={m_ten:.6e} (oracle {r_tok:.6e} {r_ten:.6e})")
        assert choice == int(ref_choice)
        np.testing.assert_allclose([m_tok, m_ten], [r_tok, r_ten], rtol=1e-10)
        per_token = bool(choice)
        del ws
    check_full_size_layer(hot, cfg, xd, wd, gyd, per_token, f"{name}.{layer.name}")


@pytest.mark.parametrize("name,idx", [("cfg3_vitb_block_b256", 1), ("cfg5_vitl_chain", 1), ("cfg4_llm7b_mlp", 1)])
def test_full_size_layers_per_tensor_quantiser(name, idx):
    """The other outcome of the quantiser selection at full size: one scale for the whole
    rotated g_y (one more pass over g_y on the separate path, a tensor-wide maximum in the
    shared passes)."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS[name]
    layer = wl.layers[idx]
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    xd, wd, gyd = hot_inputs.make_layer(wl, layer, seed=0, device="cuda")
    check_full_size_layer(hot, cfg, xd, wd, gyd, False, f"{name}.{layer.name} per-tensor")


def test_config5_chain_slice_at_full_size():
    """Three consecutive layers from the top of the ViT-L chain at 201728 tokens, as the
    benchmark's sweep runs them: each layer's g_x (as the GPU produced it) is the g_y of the
    layer below, and the oracle's stages of that layer are computed from exactly those bits."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg5_vitl_chain"]
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    fc1, fc2 = wl.layers
    depth = int(wl.extra["depth"])
    gyd = None
    for name, layer in ((f"{depth - 1}.fc2", fc2), (f"{depth - 1}.fc1", fc1), (f"{depth - 2}.fc2", fc2)):
        tag = f"{wl.name}.{name}"
        xd = hot_inputs.make_x(wl.x_kind, layer.L, layer.I, 0, tag, "cuda")
        wd = hot_inputs.make_w(layer.O, layer.I, 0, tag, "cuda")
        if gyd is None:
            gyd = hot_inputs.make_gy(wl.gy_kind, layer.L, layer.O, 0, tag, "cuda")
        assert tuple(gyd.shape) == (layer.L, layer.O)
        gx, gw = check_full_size_layer(hot, cfg, xd, wd, gyd, True, tag, one_call_strategies=(0,))
        assert torch.isfinite(gx).all().item() and gx.abs().max().item() > 0
        del xd, wd
        gyd = gx


def test_config2_per_sample_tiling_at_full_size():
    """configs[1] with its 64 samples of 197 tokens tiled separately (12 blocks of 16 and a
    padded one of 5 per sample would be n = 16; here n = 32: 6 blocks and one of 5 tokens), as
    `bench.py --sample-tokens 197` times it: INT8 and bfloat16 g_w operands, every element."""
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg2_vitb_fc1"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep, sample_tokens=197)
    ref, gw = check_gw(hot, cfg, gy, x, "cfg2 per-sample")
    check_gw_bf16(hot, hot.Config(block=wl.block, keep=wl.keep, sample_tokens=197, gw_bits=16), gy, x,
                  "cfg2 per-sample bf16")
    # the one-call form, as the benchmark calls it
    L, O = gy.shape
    I = w.shape[1]
    ws = hot.alloc_workspace(cfg, L, O, I)
    act = hot.alloc_act_buffer(cfg, L, I)
    gx1, gw1 = torch.empty((L, I), device="cuda"), torch.empty((O, I), device="cuda")
    hot.hot_compress_activation(cfg, x.cuda(), act, ws)
    hot.hot_linear_backward(cfg, gy.cuda(), w.cuda(), act, hot.HOT_Q_PER_TOKEN, gx1, gw1, ws)
    torch.cuda.synchronize()
    assert torch.equal(gw1, gw)
    ref_x = oracle.backward_gx(gy.numpy(), w.numpy(), wl.block, per_token=True)
    assert_close_maxnorm(gx1.cpu().numpy(), ref_x["g_x"], "cfg2 per-sample one call g_x")


# ---- one-call backward: both gradients from shared reads of g_y --------------------

def check_fused(hot, cfg, gy, x, w, per_token, what):
    """hot_linear_backward against the oracle's two paths, stage by stage."""
    L, O = gy.shape
    I = w.shape[1]
    _say(f"[fused] {what} L={L} O={O} I={I} n={cfg.block} r={cfg.keep} keep={cfg.keep_idx} "
         f"bits={cfg.gx_bits} token={per_token} round={cfg.rounding}")
    keep = None if cfg.keep_idx is None else list(cfg.keep_idx)
    ref_x = oracle.backward_gx(gy.numpy(), w.numpy(), cfg.block, bits=cfg.gx_bits, per_token=per_token,
                               rounding=cfg.rounding)
    codes_ref, sx_ref = oracle.compress_activation(x.numpy(), cfg.block, cfg.keep, keep=keep,
                                                   rounding=cfg.rounding)
    ref_w = oracle.backward_gw(gy.numpy(), codes_ref, sx_ref, cfg.block, cfg.keep, keep=keep,
                               rounding=cfg.rounding)
    assert ref_x["overflow"] == 0 and ref_w["overflow"] == 0
    gyd, xd, wd = gy.cuda(), x.cuda(), w.cuda()
    act = hot.alloc_act_buffer(cfg, L, I)
    ws = hot.alloc_workspace(cfg, L, O, I)
    ws.fill_(0x5A)   # stale contents must not matter
    hot.hot_compress_activation(cfg, xd, act, ws)
    gx = torch.empty((L, I), dtype=torch.float32, device="cuda")
    gw = torch.empty((O, I), dtype=torch.float32, device="cuda")
    q = hot.HOT_Q_PER_TOKEN if per_token else hot.HOT_Q_PER_TENSOR
    hot.hot_debug_set_backward_strategy(2)      # the shared passes wherever they exist
    try:
        hot.hot_linear_backward(cfg, gyd, wd, act, q, gx, gw, ws)
        if cfg.block != 64:
            t = hot.hot_debug_fused_operands(cfg, ws, act, L, O, I, q)
    finally:
        hot.hot_debug_set_backward_strategy(0)
    if cfg.block != 64:
        torch.cuda.synchronize()
        assert bits_equal(t["sg"].cpu().numpy(), ref_x["sg"]), f"{what}: g_y scales differ"
        assert bits_equal(t["sw"].cpu().numpy(), ref_x["sw"]), f"{what}: w scale differs"
        assert np.array_equal(t["qg"].cpu().numpy(), ref_x["qg"]), f"{what}: g_y codes differ"
        assert np.array_equal(t["qw"].cpu().numpy(), ref_x["qw"]), f"{what}: w codes differ"
        assert np.array_equal(t["acc_gx"].cpu().numpy().astype(np.int64), ref_x["acc"]), f"{what}: g_x accumulators differ"
        assert bits_equal(t["sgh"].cpu().numpy(), [ref_w["sg"]]), f"{what}: HLA(g_y) scale differs"
        assert np.array_equal(t["qgh"].cpu().numpy(), ref_w["qg"]), f"{what}: HLA(g_y) codes differ"
        assert np.array_equal(t["acc_gw"].cpu().numpy().astype(np.int64), ref_w["acc"]), f"{what}: g_w accumulators differ"
    torch.cuda.synchronize()
    assert_close_maxnorm(gx.cpu().numpy(), ref_x["g_x"], what + " g_x")
    assert_close_maxnorm(gw.cpu().numpy(), ref_w["g_w"], what + " g_w")
    # and bit for bit what the two separate calls give
    gx2, gw2 = torch.empty_like(gx), torch.empty_like(gw)
    hot.hot_linear_backward_gx(cfg, gyd, wd, q, gx2, ws)
    hot.hot_linear_backward_gw(cfg, gyd, act, I, gw2, ws)
    torch.cuda.synchronize()
    assert torch.equal(gx, gx2) and torch.equal(gw, gw2), f"{what}: differs from the separate calls"
    # the library's own choice of strategy gives the same bits again
    gx3, gw3 = torch.empty_like(gx), torch.empty_like(gw)
    hot.hot_linear_backward(cfg, gyd, wd, act, q, gx3, gw3, ws)
    torch.cuda.synchronize()
    assert torch.equal(gx, gx3) and torch.equal(gw, gw3), f"{what}: differs under the default strategy"


FUSED_CASES = [
    # L, O, I, n, r, keep_idx, bits
    (16, 16, 4, 16, 8, None, 4),          # one block
    (64, 48, 24, 16, 8, None, 4),         # a third of a column tile
    (272, 144, 72, 16, 8, None, 4),       # ragged column tile, L' off the pitch
    (512, 416, 136, 32, 16, None, 4),     # several column tiles, ragged last one
    (2080, 320, 140, 32, 16, None, 4),    # ragged last row tile (65 blocks)
    (512, 384, 136, 32, 16, None, 8),     # INT8 token codes
    (240, 160, 72, 16, 3, None, 4),       # odd rank: generic kept-row list
    (256, 128, 64, 16, 4, [5, 0, 9, 14], 8),
    (256, 128, 64, 32, 32, None, 4),      # full rank in sequency order
    (1024, 192, 260, 64, 32, None, 4),    # block size without shared passes
]


@pytest.mark.parametrize("case", FUSED_CASES)
@pytest.mark.parametrize("per_token", [True, False])
def test_fused_backward_small_shapes(case, per_token):
    L, O, I, n, r, keep_idx, bits = case
    hot = _hot()
    x, w, gy = make(L, O, I, seed=21, gy_kind="tok_outlier" if per_token else "chan_outlier")
    cfg = hot.Config(block=n, keep=r, keep_idx=keep_idx, gx_bits=bits)
    check_fused(hot, cfg, gy, x, w, per_token, "fused small")


def test_fused_backward_nearest_rounding_and_zero_tokens():
    hot = _hot()
    x, w, gy = make(192, 256, 96, seed=22)
    gy[17] = 0.0
    gy[64:96] = 0.0     # a whole block of zero tokens
    check_fused(hot, hot.Config(block=32, keep=16, rounding=0), gy, x, w, True, "fused rne zeros")
    check_fused(hot, hot.Config(block=16, keep=8), torch.zeros(64, 64), x[:64], w[:64], False, "fused all zero")


def test_fused_backward_config1_full():
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg1_single_512x768x768"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    check_fused(hot, hot.Config(block=wl.block, keep=wl.keep), gy, x, w, True, "fused cfg1")


# ---- frozen weights: H.w quantised once, g_x only (Sec. 5.3) -------------------------

@pytest.mark.parametrize("n,bits,per_token,shape", [(16, 4, True, (264, 448, 136)), (32, 4, False, (264, 448, 136)),
                                                    (64, 8, True, (264, 448, 136)),
                                                    # few output tiles, long K: the GEMM splits K and its
                                                    # scratch follows the g_y codes in the smaller workspace
                                                    (16, 4, True, (264, 2048, 384)), (32, 8, False, (300, 2048, 200))])
def test_frozen_weight_gx_matches_oracle_and_uncached_call(n, bits, per_token, shape):
    hot = _hot()
    L, O, I = shape
    x, w, gy = make(L, O, I, seed=31)
    cfg = hot.Config(block=n, keep=n // 2, gx_bits=bits)
    _say(f"[gx cached] L={L} O={O} I={I} n={n} bits={bits} token={per_token}")
    ref = oracle.backward_gx(gy.numpy(), w.numpy(), n, bits=bits, per_token=per_token, rounding=cfg.rounding)
    q = hot.HOT_Q_PER_TOKEN if per_token else hot.HOT_Q_PER_TENSOR
    wd = w.cuda()
    ws0 = hot.alloc_workspace(cfg, L, O, I)
    wq = hot.alloc_weight_buffer(cfg, O, I)
    hot.hot_quantize_weight(cfg, wd, wq, ws0[:hot.HOT_WS_PREFIX_BYTES])
    codes, sw = hot.hot_debug_unpack_weight(cfg, wq, O, I)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), ref["qw"]) and bits_equal(sw.cpu().numpy(), ref["sw"])
    # the cached call's own, smaller workspace, placed so that anything written past its end
    # lands in a guard region
    need = hot.hot_gx_cached_workspace_bytes(cfg, L, O, I)
    assert 0 < need <= ws0.numel() - O * I * bits // 8
    guarded = torch.full((need + 4096,), 0x33, dtype=torch.uint8, device="cuda")
    ws = guarded[:need]
    gx = torch.empty((L, I), device="cuda")
    for step in range(2):   # second step: another g_y against the same cached weights
        g = gy if step == 0 else hot_inputs.make_gy("t4", L, O, 32, "step2")
        r = ref if step == 0 else oracle.backward_gx(g.numpy(), w.numpy(), n, bits=bits, per_token=per_token,
                                                     rounding=cfg.rounding)
        hot.hot_linear_backward_gx_cached(cfg, g.cuda(), wq, I, q, gx, ws)
        torch.cuda.synchronize()
        assert (guarded[need:] == 0x33).all().item(), "written past the documented workspace size"
        ws0[:need].copy_(ws)    # the operand view decodes a full-size workspace
        taps = hot.hot_debug_gx_operands(cfg, ws0, L, O, I, q, want_acc=False)
        torch.cuda.synchronize()
        assert np.array_equal(taps["qg"].cpu().numpy(), r["qg"]) and bits_equal(taps["sg"].cpu().numpy(), r["sg"])
        assert_close_maxnorm(gx.cpu().numpy(), r["g_x"], f"cached g_x step {step}")
        gx2 = torch.empty_like(gx)
        ws2 = hot.alloc_workspace(cfg, L, O, I)
        hot.hot_linear_backward_gx(cfg, g.cuda(), wd, q, gx2, ws2)
        torch.cuda.synchronize()
        assert torch.equal(gx, gx2)


# ---- column quantiser: single-pass and two-pass kernels must agree with the oracle ----

@pytest.fixture
def exchange_wait():
    hot = _hot()
    yield hot.hot_debug_set_exchange_wait_us
    hot.hot_debug_set_exchange_wait_us(200)


@pytest.mark.parametrize("wait_us", [-1, 0, 200])
def test_column_quantiser_paths(exchange_wait, wait_us):
    """wait < 0: two-pass kernels; 0: single pass where every workgroup computes the other
    workgroups' maxima itself (what happens when they are late); 200: the default."""
    hot = _hot()
    exchange_wait(wait_us)
    for (L, O, I, n, r, keep_idx) in [(272, 130, 72, 16, 8, None), (2048, 300, 140, 16, 8, None),
                                      (1024, 224, 260, 32, 16, None), (1024, 96, 260, 64, 32, None),
                                      (240, 64, 72, 16, 3, None), (256, 64, 64, 16, 4, [5, 0, 9, 14])]:
        x, w, gy = make(L, O, I, seed=41)
        cfg = hot.Config(block=n, keep=r, keep_idx=keep_idx)
        check_gw(hot, cfg, gy, x, f"wait={wait_us}")
        if O % n == 0:
            check_gx(hot, cfg, gy, w, True, f"wait={wait_us}")
            check_gx(hot, hot.Config(block=n, keep=r, keep_idx=keep_idx, gx_bits=8), gy, w, False, f"wait={wait_us}")


def test_single_pass_16_row_blocks_with_an_odd_block_count():
    """16-row blocks leave 8 code bytes per block and column, which the single-pass kernel
    stores two blocks at a time; with an odd number of blocks the last pair's second half is
    the row's zero padding (checked through the GEMM, which reads the padding as K)."""
    hot = _hot()
    L, O, I = 16 * 3151, 48, 768
    x, w, gy = make(L, O, I, seed=43)
    check_gw(hot, hot.Config(block=16, keep=8), gy, x, "odd block count")


def test_single_pass_transposed_stores_with_ragged_edges():
    """Runs of 64 code bytes or more per lane leave the single-pass kernel through a
    wave-private transposition (a store instruction then writes whole runs of an output row).
    Shapes that take that path (4 blocks per wave of 32 rows, 8 of 16 rows) with a last column
    tile that is partly empty and a last row tile that holds a single block: every code, the
    padding (through the GEMM, which reads it as K) and the scale must be the oracle's."""
    hot = _hot()
    for (n, L, O, I, seed) in [(32, 32 * 385, 200, 1000, 51), (16, 16 * 1443, 48, 1000, 52)]:
        x, w, gy = make(L, O, I, seed=seed)
        check_gw(hot, hot.Config(block=n, keep=n // 2), gy, x, f"transposed stores n={n}")
    # the weight operand of the g_x path (INT4, all rows kept): 2592 x 4040, few tokens
    x, w, gy = make(64, 2592, 4040, seed=53)
    check_gx(hot, hot.Config(block=32, keep=16), gy, w, True, "transposed stores, weights")
    check_gx(hot, hot.Config(block=32, keep=16), gy, w, False, "transposed stores, weights, per tensor")


def test_config2_two_pass_column_kernels(exchange_wait):
    """configs[1] with the single-pass kernels switched off (x and w then take the same
    two-pass kernels as tensors too large for the register files)."""
    hot = _hot()
    exchange_wait(-1)
    wl = hot_inputs.WORKLOADS["cfg2_vitb_fc1"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    check_gx(hot, cfg, gy, w, True, "cfg2 two-pass")
    check_gw(hot, cfg, gy, x, "cfg2 two-pass")


def test_gx_combined_and_separate_launches_agree():
    """By default small weights and the per-token g_y operand are quantised in one launch;
    strategy 3 gives every kernel its own launch.  Codes, scales and g_x must be the same
    bits, with the exchange of the weight workgroups both waited for and skipped."""
    hot = _hot()
    try:
        # O at both ends of every row-kernel variant the combined launch has (257..4096), token
        # counts that leave the last 4-row workgroup partly empty, weights of one tile and of
        # hundreds, and shapes just outside (O = 256, 4160: separate launches either way)
        for (L, O, I, n) in [(2048, 768, 768, 32), (1024, 3072, 768, 32), (788, 512, 1024, 16), (4096, 4096, 256, 64),
                             (512, 1024, 128, 16), (1030, 272, 64, 16), (777, 1040, 72, 16), (130, 2048, 66, 32),
                             (96, 256, 64, 32), (64, 4160, 32, 32)]:
            x, w, gy = make(L, O, I, seed=53)
            cfg = hot.Config(block=n, keep=n // 2)
            outs = []
            for strategy, wait in [(0, 200), (3, 200), (0, 0)]:
                hot.hot_debug_set_backward_strategy(strategy)
                hot.hot_debug_set_exchange_wait_us(wait)
                ref, gx = check_gx(hot, cfg, gy, w, True, f"strategy={strategy} wait={wait}")
                outs.append(gx.clone())
            assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    finally:
        hot.hot_debug_set_backward_strategy(0)
        hot.hot_debug_set_exchange_wait_us(200)


# ---- GEMM work distribution: one workgroup per tile and K splits must give the same integers ----

@pytest.fixture
def gemm_mode():
    hot = _hot()
    yield hot.hot_debug_set_gemm_mode
    hot.hot_debug_set_gemm_mode(0)
    hot.hot_debug_set_exchange_wait_us(200)


@pytest.mark.parametrize("mode,wait_us", [(1, 200), (2, 200), (3, 200), (8, 200), (2, 0), (5, 0),
                                          (10, 200), (11, 200), (12, 200), (13, 200)])
def test_gemm_work_distribution(gemm_mode, mode, wait_us):
    """mode 1: a workgroup per output tile; mode s >= 2: K cut into s slices whose
    workgroups hand partial sums to the tile's last one through the workspace; wait 0: no
    owner ever waits, every missing slice is computed by the owner itself (what happens when
    the other workgroup is late); modes 10-13: every GEMM on one given tile shape (128x128,
    192x256, 256x256, 128x256), whatever the planner would pick.  Shapes: few tiles with long
    K, many tiles, ragged tiles (interior tiles take the unchecked epilogue, edge tiles the
    checked one), K too short to split."""
    hot = _hot()
    gemm_mode(mode)
    hot.hot_debug_set_exchange_wait_us(wait_us)
    for (L, O, I, n, r) in [(2048, 300, 140, 16, 8), (8192, 256, 128, 32, 16), (4096, 1056, 520, 32, 16),
                            (512, 96, 80, 32, 16), (16384, 64, 64, 16, 8)]:
        x, w, gy = make(L, O, I, seed=43)
        cfg = hot.Config(block=n, keep=r)
        check_gw(hot, cfg, gy, x, f"gemm mode={mode} wait={wait_us}")
        if O % n == 0:
            check_gx(hot, cfg, gy, w, True, f"gemm mode={mode} wait={wait_us}")
            check_gx(hot, hot.Config(block=n, keep=r, gx_bits=8), gy, w, False, f"gemm mode={mode} wait={wait_us}")


@pytest.mark.parametrize("mode,wait_us", [(3, 200), (4, 0)])
def test_config2_split_k(gemm_mode, mode, wait_us):
    hot = _hot()
    gemm_mode(mode)
    hot.hot_debug_set_exchange_wait_us(wait_us)
    wl = hot_inputs.WORKLOADS["cfg2_vitb_fc1"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep)
    check_gx(hot, cfg, gy, w, True, "cfg2 split-K")
    check_gw(hot, cfg, gy, x, "cfg2 split-K")


def test_int8_gemm_on_the_large_tile():
    """Shapes for which the INT8 GEMMs take the 256x256 tile (eight waves per workgroup), with
    ragged edges in both directions: the g_w GEMM of a 2200 x 2100 weight and the INT8 g_x
    GEMM of 4000 tokens; every accumulator is compared."""
    hot = _hot()
    x, w, gy = make(8192, 2200, 2100, seed=71)     # K = 4096 bytes: long enough for the planner
    check_gw(hot, hot.Config(block=16, keep=8), gy, x, "large INT8 tile, g_w")
    x, w, gy = make(4000, 8192, 1100, seed=72)
    check_gx(hot, hot.Config(block=16, keep=8, gx_bits=8), gy, w, False, "large INT8 tile, g_x")
    check_gx(hot, hot.Config(block=16, keep=8, gx_bits=8), gy, w, True, "large INT8 tile, g_x")


def test_bf16_gemm_on_the_large_tile():
    """The bfloat16 g_w GEMM of a 2200 x 2100 weight takes the 256x256 tile (eight waves)."""
    hot = _hot()
    x, w, gy = make(8192, 2200, 2100, seed=74)
    check_gw_bf16(hot, hot.Config(block=16, keep=8, gw_bits=16), gy, x, "large bf16 tile")


@pytest.mark.parametrize("wait_us", [200, 0])
def test_int8_gemm_large_tile_with_k_split(gemm_mode, wait_us):
    """A small output with a very long K (40000 reduced tokens): the g_w GEMM takes the 256x256
    tile with K in two slices; with wait 0 the owner computes the other slice itself."""
    hot = _hot()
    hot.hot_debug_set_exchange_wait_us(wait_us)
    x, w, gy = make(80000, 300, 260, seed=73)
    check_gw(hot, hot.Config(block=16, keep=8), gy, x, f"large INT8 tile, K split, wait={wait_us}")


def test_split_k_hand_over_sees_fresh_partial_sums(gemm_mode):
    """Two different inputs alternate through the same workspace, twelve back-to-back steps
    without a host synchronisation in between: every g_w must equal the one computed without
    a K split for that input.  A partial sum left in some cache by an earlier launch, or a
    flag of an earlier launch taken for a fresh one, would show up here."""
    hot = _hot()
    L, O, I = 8192, 384, 256          # 6 tiles of 128x128, K of 32 stages: split in 8
    cfg = hot.Config(block=32, keep=16)
    data = [make(L, O, I, seed=61), make(L, O, I, seed=62)]
    ws = hot.alloc_workspace(cfg, L, O, I)
    acts, want = [], []
    gemm_mode(1)
    for x, w, gy in data:
        act = hot.alloc_act_buffer(cfg, L, I)
        hot.hot_compress_activation(cfg, x.cuda(), act, ws)
        gw = torch.empty((O, I), device="cuda")
        hot.hot_linear_backward_gw(cfg, gy.cuda(), act, I, gw, ws)
        torch.cuda.synchronize()
        acts.append(act)
        want.append(gw.clone())
    assert not torch.equal(want[0], want[1])
    gemm_mode(0)
    gys = [d[2].cuda() for d in data]
    outs = [torch.empty((O, I), device="cuda") for _ in range(12)]
    for step in range(12):
        hot.hot_linear_backward_gw(cfg, gys[step % 2], acts[step % 2], I, outs[step], ws)
    torch.cuda.synchronize()
    for step in range(12):
        assert torch.equal(outs[step], want[step % 2]), f"step {step}"


# ---- maximum reduction lengths: accumulators at the edge of int32 ------------------------

def _hadamard_np(n):
    H = np.array([[1.0]])
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H


def test_gx_longest_reduction_with_saturated_codes():
    """O at the documented limit with every code of both operands equal to +7 (inputs are
    H t / n per block, so the rotated values are the constant t exactly): the INT4 operands
    are fed to the matrix cores as 16 x code, so the internal sum 256 * 49 * O must still
    fit int32, and the true accumulator is 49 * O everywhere."""
    hot = _hot()
    n, O, L, I = 64, 171136, 3, 5
    assert O % n == 0 and 256 * 49 * O < 2 ** 31 <= 256 * 49 * (O + n)
    H = _hadamard_np(n)
    blk_g = (H @ np.full(n, 0.5)) / n           # exact: small dyadic values
    blk_w = (H @ np.full(n, 0.25)) / n
    gy = torch.from_numpy(np.tile(blk_g, (L, O // n)).astype(np.float32))
    w = torch.from_numpy(np.tile(blk_w.reshape(n, 1), (O // n, I)).astype(np.float32))
    cfg = hot.Config(block=n, keep=n // 2)
    for per_token in (True, False):
        ref, gx = check_gx(hot, cfg, gy, w, per_token, "longest O")
        assert (ref["qg"] == 7).all() and (ref["qw"] == 7).all() and (ref["acc"] == 49 * O).all()


def test_gw_longest_reduction_with_saturated_codes():
    """L' at the documented limit with every INT8 code of both operands equal to +127:
    127^2 * L' is the largest accumulator the g_w path can produce."""
    hot = _hot()
    n, r, O, I = 16, 8, 16, 16
    Lr = 133120
    L = Lr * n // r
    assert 127 * 127 * Lr < 2 ** 31 and Lr <= 133144 < Lr + 128
    H = _hadamard_np(n)
    t = np.zeros(n)
    t[oracle.lowpass_index(n, r)] = 2.0          # kept rows carry the constant, dropped rows 0
    blk = (H @ t) / n
    gy = torch.from_numpy(np.tile(blk.reshape(n, 1), (L // n, O)).astype(np.float32))
    x = torch.from_numpy(np.tile((blk * 3.0).reshape(n, 1), (L // n, I)).astype(np.float32))
    cfg = hot.Config(block=n, keep=r)
    ref, gw = check_gw(hot, cfg, gy, x, "longest L'")
    assert (ref["qg"] == 127).all() and (ref["acc"] == 127 * 127 * Lr).all()


# ---- bfloat16 variant of the g_w path (gw_bits = 16) ----------------------------------------

def check_gw_bf16(hot, cfg, gy, x, what):
    """Operand bit patterns must be identical; fp32 accumulators and g_w within 1e-5 of the
    oracle's double-precision sum of the same bf16 products (max-norm)."""
    L, O = gy.shape
    I = x.shape[1]
    n, r = cfg.block, cfg.keep
    _say(f"[gw bf16] {what} L={L} O={O} I={I} n={n} r={r} keep={cfg.keep_idx}")
    keep = None if cfg.keep_idx is None else list(cfg.keep_idx)
    S = cfg.sample_tokens
    xo = oracle.pad_samples(x.numpy(), S, n) if S else x.numpy()
    gyo = oracle.pad_samples(gy.numpy(), S, n) if S else gy.numpy()
    xb_ref = oracle.compress_activation_bf16(xo, n, r, keep)
    ref = oracle.backward_gw_bf16(gyo, xb_ref, n, r, keep)
    gyd, xd = gy.cuda(), x.cuda()
    act = hot.alloc_act_buffer(cfg, L, I)
    ws = hot.alloc_workspace(cfg, L, O, I)
    ws.fill_(0x5A)
    hot.hot_compress_activation(cfg, xd, act, ws)
    codes, sx = hot.hot_debug_unpack_activation(cfg, act, L, I)
    gw = torch.empty((O, I), dtype=torch.float32, device="cuda")
    hot.hot_linear_backward_gw(cfg, gyd, act, I, gw, ws)
    taps = hot.hot_debug_gw_operands(cfg, ws, act, L, O, I)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy().view(np.uint16), xb_ref), f"{what}: bf16 activation differs"
    assert np.array_equal(taps["qg"].cpu().numpy().view(np.uint16), ref["gh_bits"]), f"{what}: bf16 HLA(g_y) differs"
    assert sx.item() == 1.0 and taps["sg"].item() == 1.0
    assert_close_maxnorm(taps["acc"].cpu().numpy(), ref["g_w"] * n, what + " accumulators", exact_accumulators=False)
    assert_close_maxnorm(gw.cpu().numpy(), ref["g_w"], what + " g_w", exact_accumulators=False)
    Lr = cfg.reduced_tokens(L)
    assert hot.hot_act_buffer_bytes(cfg, L, I) == 256 + I * ((2 * Lr + 127) // 128 * 128)
    return ref, gw


@pytest.mark.parametrize("case", [(16, 8, 4, 16, 8, None), (272, 130, 72, 16, 8, None),
                                  (512, 200, 136, 32, 16, None), (1024, 96, 260, 64, 32, None),
                                  (240, 64, 72, 16, 3, None), (256, 64, 64, 16, 4, [5, 0, 9, 14]),
                                  (256, 64, 64, 16, 16, None), (4096, 300, 140, 16, 8, None)])
def test_gw_bf16_small_shapes(case):
    L, O, I, n, r, keep_idx = case
    hot = _hot()
    x, w, gy = make(L, O, I, seed=51, gy_kind="t4")
    check_gw_bf16(hot, hot.Config(block=n, keep=r, keep_idx=keep_idx, gw_bits=16), gy, x, "bf16 small")


def test_gw_bf16_config2_full_size():
    hot = _hot()
    wl = hot_inputs.WORKLOADS["cfg2_vitb_fc1"]
    x, w, gy = hot_inputs.make_layer(wl, wl.layers[0], seed=0)
    cfg = hot.Config(block=wl.block, keep=wl.keep, gw_bits=16)
    ref, gw = check_gw_bf16(hot, cfg, gy, x, "bf16 cfg2")
    _, exact = oracle.exact_backward(gy.numpy(), x.numpy(), w.numpy(), want_gx=False)
    rel = np.linalg.norm(gw.cpu().numpy() - exact) / np.linalg.norm(exact)
    _say(f"cfg2 bf16 g_w relative Frobenius error vs exact backward (statistic): {rel:.4f}")
    # the one-call form takes the same path for its g_w half
    gx = torch.empty((gy.shape[0], w.shape[1]), device="cuda")
    gw2 = torch.empty_like(gw)
    ws = hot.alloc_workspace(cfg, *gy.shape, w.shape[1])
    act = hot.alloc_act_buffer(cfg, gy.shape[0], x.shape[1])
    hot.hot_compress_activation(cfg, x.cuda(), act, ws)
    hot.hot_linear_backward(cfg, gy.cuda(), w.cuda(), act, hot.HOT_Q_PER_TOKEN, gx, gw2, ws)
    torch.cuda.synchronize()
    assert torch.equal(gw, gw2)


# ---- per-sample tiling of the token axis (sample_tokens > 0) ---------------------------------

RAGGED_CASES = [
    # B, S, O, I, n, r, keep_idx
    (4, 197, 130, 72, 16, 8, None),       # ViT sequence: 12 blocks + one of 5 tokens
    (3, 197, 96, 40, 32, 16, None),
    (2, 197, 64, 24, 64, 32, None),
    (5, 10, 48, 16, 16, 8, None),         # samples shorter than a block
    (6, 64, 40, 24, 16, 8, None),         # multiple of the block: same result as one run
    (4, 50, 33, 20, 16, 3, None),         # generic kept list
    (16, 197, 200, 136, 16, 8, None),     # several row tiles
]


@pytest.mark.parametrize("case", RAGGED_CASES)
@pytest.mark.parametrize("wait_us", [-1, 0, 200])
def test_gw_per_sample_tiling(exchange_wait, case, wait_us):
    B, S, O, I, n, r, keep_idx = case
    hot = _hot()
    exchange_wait(wait_us)
    x, w, gy = make(B * S, O, I, seed=61)
    cfg = hot.Config(block=n, keep=r, keep_idx=keep_idx, sample_tokens=S)
    ref, gw = check_gw(hot, cfg, gy, x, f"per-sample S={S} wait={wait_us}")
    if S % n == 0:
        flat = hot.Config(block=n, keep=r, keep_idx=keep_idx)
        _, gw_flat = check_gw(hot, flat, gy, x, "same tokens as one run")
        assert torch.equal(gw, gw_flat)
    if wait_us == 200:
        check_gw_bf16(hot, hot.Config(block=n, keep=r, keep_idx=keep_idx, gw_bits=16, sample_tokens=S),
                      gy, x, f"per-sample bf16 S={S}")


def test_per_sample_tiling_shape_errors_and_gx_is_unaffected():
    hot = _hot()
    cfg = hot.Config(block=16, keep=8, sample_tokens=197)
    assert hot.hot_act_buffer_bytes(cfg, 4 * 197, 64) == 256 + 64 * ((4 * 13 * 8 + 127) // 128 * 128)
    assert hot.hot_act_buffer_bytes(cfg, 4 * 197 + 1, 64) == 0      # not a whole number of samples
    x, w, gy = make(2 * 197, 64, 24, seed=62)
    check_gx(hot, cfg, gy, w, True, "g_x with sample_tokens set")     # L need not be a multiple of n


# ---- calls recorded into a HIP graph ----------------------------------------------------------------

def test_replayable_calls_in_a_hip_graph():
    """With hot_config.replayable the launch tags come from an epoch in the workspace that every
    call advances, so a recorded step can be replayed.  One step of configs[0] (compression, both
    gradients: single-pass exchange kernels, the combined weight / g_y launch and the split-K g_w
    GEMM, all of which use tags) is captured once and replayed six times on inputs that change
    between the replays, with eager work and a synchronisation in between; every replay must
    give the bits of the eager, host-tagged call on the same inputs, and the first also the
    oracle's.  Half of the replays run with the exchange wait at zero, so that workgroups also
    take the path that recomputes the other tiles' maxima."""
    hot = _hot()
    L, O, I = 512, 768, 768
    cfg_r = hot.Config(block=16, keep=8, replayable=True)
    cfg_e = hot.Config(block=16, keep=8)
    dev = "cuda"
    xs, ws_, gys = zip(*[make(L, O, I, seed=70 + k, gy_kind=("chan_outlier", "tok_outlier", "normal")[k % 3])
                         for k in range(7)])
    x_d, w_d, gy_d = xs[0].to(dev), ws_[0].to(dev), gys[0].to(dev)
    act_r, work_r = hot.alloc_act_buffer(cfg_r, L, I), hot.alloc_workspace(cfg_r, L, O, I)
    act_e, work_e = hot.alloc_act_buffer(cfg_e, L, I), hot.alloc_workspace(cfg_e, L, O, I)
    gx_r, gw_r = torch.empty((L, I), device=dev), torch.empty((O, I), device=dev)
    gx_e, gw_e = torch.empty((L, I), device=dev), torch.empty((O, I), device=dev)

    def step(cfg, act, work, gx, gw):
        hot.hot_compress_activation(cfg, x_d, act, work)
        hot.hot_linear_backward(cfg, gy_d, w_d, act, hot.HOT_Q_PER_TOKEN, gx, gw, work)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # launch plans are made on first use: once before recording
        step(cfg_r, act_r, work_r, gx_r, gw_r)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(cfg_r, act_r, work_r, gx_r, gw_r)
    torch.cuda.synchronize()
    try:
        for k in range(1, 7):
            _say(f"[graph] replay {k}")
            hot.hot_debug_set_exchange_wait_us(0 if k % 2 == 0 else 200)
            x_d.copy_(xs[k].to(dev)); w_d.copy_(ws_[k].to(dev)); gy_d.copy_(gys[k].to(dev))   # eager work
            gx_r.fill_(float("nan")); gw_r.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            step(cfg_e, act_e, work_e, gx_e, gw_e)
            torch.cuda.synchronize()
            codes_r, sx_r = hot.hot_debug_unpack_activation(cfg_r, act_r, L, I)
            codes_e, sx_e = hot.hot_debug_unpack_activation(cfg_e, act_e, L, I)
            assert torch.equal(codes_r, codes_e) and torch.equal(sx_r, sx_e), \
                f"replay {k}: compressed activation differs from the eager call"
            assert torch.equal(gx_r, gx_e), f"replay {k}: g_x differs from the eager call"
            assert torch.equal(gw_r, gw_e), f"replay {k}: g_w differs from the eager call"
            if k == 1:
                ref_codes, ref_sx = oracle.compress_activation(xs[k].numpy(), 16, 8)
                ref_x = oracle.backward_gx(gys[k].numpy(), ws_[k].numpy(), 16, bits=4, per_token=True)
                ref_w = oracle.backward_gw(gys[k].numpy(), ref_codes, ref_sx, 16, 8)
                assert_close_maxnorm(gx_r.cpu().numpy(), ref_x["g_x"], "replayed g_x")
                assert_close_maxnorm(gw_r.cpu().numpy(), ref_w["g_w"], "replayed g_w")
    finally:
        hot.hot_debug_set_exchange_wait_us(200)


def test_replayable_calls_give_the_bits_of_host_tagged_calls():
    """Every entry point that launches tagged kernels, with tags from the workspace epoch and
    with tags from the host: the same bits, on a shape whose g_w GEMM splits K and whose
    transforms take the single-pass kernels (the g_x call twice in a row, so that the second
    call finds the first one's slots and flags in the workspace)."""
    hot = _hot()
    L, O, I = 1024, 768, 512
    x, w, gy = make(L, O, I, seed=81)
    xd, wd, gyd = x.cuda(), w.cuda(), gy.cuda()
    outs = {}
    for replayable in (False, True):
        cfg = hot.Config(block=16, keep=8, replayable=replayable)
        ws = hot.alloc_workspace(cfg, L, O, I)
        act, wq = hot.alloc_act_buffer(cfg, L, I), hot.alloc_weight_buffer(cfg, O, I)
        g = {k: torch.empty((L, I), device="cuda") for k in ("gx", "gx2", "cached", "noalloc", "both_x")}
        gw, gw2 = torch.empty((O, I), device="cuda"), torch.empty((O, I), device="cuda")
        hot.hot_compress_activation(cfg, xd, act, ws)
        hot.hot_linear_backward_gx(cfg, gyd, wd, hot.HOT_Q_PER_TOKEN, g["gx"], ws)
        hot.hot_linear_backward_gx(cfg, gyd, wd, hot.HOT_Q_PER_TENSOR, g["gx2"], ws)
        hot.hot_quantize_weight(cfg, wd, wq, ws)
        hot.hot_linear_backward_gx_cached(cfg, gyd, wq, I, hot.HOT_Q_PER_TOKEN, g["cached"], ws)
        hot.hot_linear_backward_gx_noalloc(cfg, gyd, wd, hot.HOT_Q_PER_TOKEN, g["noalloc"])
        hot.hot_linear_backward_gw(cfg, gyd, act, I, gw, ws)
        hot.hot_linear_backward(cfg, gyd, wd, act, hot.HOT_Q_PER_TOKEN, g["both_x"], gw2, ws)
        torch.cuda.synchronize()
        outs[replayable] = {**{k: v.cpu() for k, v in g.items()}, "gw": gw.cpu(), "gw2": gw2.cpu()}
    for k in outs[False]:
        assert torch.equal(outs[False][k], outs[True][k]), f"{k}: replayable call differs from the host-tagged call"
    assert torch.equal(outs[True]["gx"], outs[True]["cached"]) and torch.equal(outs[True]["gx"], outs[True]["noalloc"])
    assert torch.equal(outs[True]["gx"], outs[True]["both_x"]) and torch.equal(outs[True]["gw"], outs[True]["gw2"])
    ref = oracle.backward_gx(gy.numpy(), w.numpy(), 16, bits=4, per_token=True)
    assert_close_maxnorm(outs[True]["gx"].numpy(), ref["g_x"], "replayable g_x")


# ---- seeded random shapes and settings ----------------------------------------------------------

def test_seeded_random_shapes_and_settings(exchange_wait, gemm_mode):
    """120 small cases drawn with a fixed seed: block size, rank, kept-row list, per-sample
    tiling, code widths, quantiser, rounding, column-kernel path (two-pass / single pass with
    or without waiting) and GEMM work distribution, each against the oracle stage by stage."""
    import random
    hot = _hot()
    rnd = random.Random(20250)
    for it in range(120):
        n = rnd.choice([16, 16, 32, 32, 64])
        mode = rnd.choice(["gx", "gw", "fused", "gw", "gx"])
        r = rnd.choice([1, 2, 3, n // 4, n // 2, n // 2, n // 2, n, rnd.randint(1, n)])
        keep_idx = rnd.sample(range(n), r) if rnd.random() < 0.2 else None
        S = 0
        if mode == "gx":
            L = rnd.randint(1, 1500)
        elif mode == "gw" and rnd.random() < 0.3:
            S = rnd.randint(1, 200)
            L = S * rnd.randint(1, 8)
        else:
            L = n * rnd.randint(1, 60)
        O = n * rnd.randint(1, 24) if mode in ("gx", "fused") else rnd.randint(1, 600)
        I = rnd.randint(1, 400)
        per_token = rnd.random() < 0.6
        cfg = hot.Config(block=n, keep=r, keep_idx=keep_idx, gx_bits=rnd.choice([4, 4, 8]),
                         rounding=rnd.choice([0, 1, 1]), sample_tokens=S)
        wait_us, mode_g = rnd.choice([-1, 0, 200, 200]), rnd.choice([0, 0, 1, 2, 5])
        x, w, gy = make(L, O, I, seed=1000 + it, gy_kind=rnd.choice(["chan_outlier", "tok_outlier", "normal"]))
        exchange_wait(wait_us)
        gemm_mode(mode_g)
        what = f"random case {it} wait={wait_us} gemm={mode_g}"
        if mode == "gx":
            check_gx(hot, cfg, gy, w, per_token, what)
        elif mode == "gw":
            check_gw(hot, cfg, gy, x, what)
        else:
            check_fused(hot, cfg, gy, x, w, per_token, what)
