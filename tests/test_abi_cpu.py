"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function hot.h declares, sizes follow the documented layouts, and invalid
arguments are rejected before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2503_21261_amd as hot

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hot.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hot_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = hot.lib()
    names = declared_functions()
    assert set(names) == set(hot.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_default_config_is_the_papers():
    cfg = hot.hot_config()
    hot.lib().hot_default_config(C.byref(cfg))
    assert (cfg.block, cfg.keep, cfg.gx_bits, cfg.gw_bits, cfg.rounding) == (16, 8, 4, 8, 1)
    assert cfg.lqs_threshold == 0.5 and not cfg.keep_idx
    assert cfg.sample_tokens == 0 and cfg.replayable == 0
    d = hot.Config()
    assert (d.block, d.keep, d.gx_bits, d.gw_bits, d.rounding, d.lqs_threshold) == (16, 8, 4, 8, 1, 0.5)


def test_act_buffer_is_one_eighth_of_fp32():
    # Sec. 5.2.1: HLA r/n = 1/2 (50 %) times FP32 -> INT8 (25 %) = 12.5 %, plus the header
    cfg = hot.Config()
    for L, I in ((512, 768), (50432, 768), (201728, 1024)):
        Lr = L // 2
        pitch = (Lr + 127) // 128 * 128
        assert hot.hot_act_buffer_bytes(cfg, L, I) == 256 + pitch * I
    assert hot.hot_act_buffer_bytes(cfg, 512, 768) == 256 + 512 * 768 * 4 // 8
    assert hot.hot_act_buffer_bytes(hot.Config(block=16, keep=16), 512, 768) == 256 + 512 * 768
    assert hot.hot_act_buffer_bytes(cfg, 500, 768) == 0          # L % n != 0
    assert hot.hot_act_buffer_bytes(hot.Config(block=24), 480, 768) == 0


def test_bf16_activation_buffer_is_a_quarter_of_fp32():
    cfg = hot.Config(block=32, keep=16, gw_bits=16)
    L, I = 12608, 768
    assert hot.hot_act_buffer_bytes(cfg, L, I) == 256 + I * ((L + 127) // 128 * 128)
    # no int32 bound on the reduction length with fp32 accumulation
    assert hot.hot_act_buffer_bytes(hot.Config(gw_bits=16), 16 * 2 * 140000, 8) > 0
    assert hot.hot_act_buffer_bytes(hot.Config(gw_bits=8), 16 * 2 * 140000, 8) == 0
    assert hot.hot_workspace_bytes(hot.Config(gw_bits=12), 64, 64, 64) == 0


def test_weight_buffer_is_a_header_plus_padded_code_rows():
    assert hot.hot_weight_buffer_bytes(hot.Config(), 768, 768) == 256 + 768 * 384
    assert hot.hot_weight_buffer_bytes(hot.Config(gx_bits=8), 144, 10) == 256 + 10 * 256
    assert hot.hot_weight_buffer_bytes(hot.Config(), 100, 10) == 0


def test_workspace_covers_the_documented_operands():
    cfg = hot.Config()
    L, O, I = 512, 768, 768
    need = hot.hot_workspace_bytes(cfg, L, O, I)
    assert need >= 256 + L * 4 + L * O // 2 + I * O // 2         # g_x operands, INT4
    assert need >= 256 + O * (L // 2)                            # HLA(g_y), INT8
    assert hot.hot_workspace_bytes(hot.Config(gx_bits=8), L, O, I) >= L * O + I * O
    assert hot.hot_workspace_bytes(hot.Config(gx_bits=5), L, O, I) == 0


@pytest.mark.parametrize("bad", [dict(block=8), dict(block=48), dict(keep=0), dict(keep=17),
                                 dict(gx_bits=2), dict(gw_bits=4), dict(rounding=2),
                                 dict(keep=2, keep_idx=[3, 3]), dict(keep=2, keep_idx=[0, 16]),
                                 dict(lqs_threshold=-1.0)])
def test_bad_config_is_an_argument_error(bad):
    cfg = hot.Config(**bad)
    fake = C.c_void_p(4096)
    st = hot.lib().hot_linear_backward_gx(C.byref(cfg.c()), fake, fake, 64, 64, 64, 1, fake, fake, 1 << 30, None)
    assert st == hot.HOT_ERR_ARG
    assert hot.hot_workspace_bytes(cfg, 64, 64, 64) == 0


def test_replayable_is_a_flag():
    """hot_config.replayable is 0 or 1; anything else is refused before any launch."""
    cfg = hot.Config().c()
    fake = C.c_void_p(4096)
    for value, want in ((2, hot.HOT_ERR_ARG), (-1, hot.HOT_ERR_ARG)):
        cfg.replayable = value
        st = hot.lib().hot_linear_backward_gx(C.byref(cfg), fake, fake, 64, 64, 64, 1, fake, fake, 1 << 30, None)
        assert st == want
    cfg.replayable = 1      # accepted: the call then fails on its workspace size, still before any launch
    assert hot.lib().hot_linear_backward_gx(C.byref(cfg), fake, fake, 64, 64, 64, 1, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE


def test_argument_shape_and_workspace_errors_precede_any_launch():
    lib, cfg = hot.lib(), hot.Config()
    c = C.byref(cfg.c())
    fake = C.c_void_p(4096)      # never dereferenced: every call below fails its host checks
    big = 1 << 40
    assert lib.hot_linear_backward_gx(c, None, fake, 64, 64, 64, 1, fake, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_linear_backward_gx(c, C.c_void_p(4100), fake, 64, 64, 64, 1, fake, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_linear_backward_gx(c, fake, fake, 64, 64, 64, 7, fake, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_linear_backward_gx(c, fake, fake, 64, 72, 64, 1, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward_gx(c, fake, fake, 0, 64, 64, 1, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward_gx(c, fake, fake, 64, 171200, 64, 1, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward_gx(c, fake, fake, 64, 64, 64, 1, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE
    assert lib.hot_linear_backward_gw(c, fake, fake, 72, 64, 64, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward_gw(c, fake, fake, 16 * 2 * 133152, 64, 64, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward_gw(c, fake, fake, 64, 64, 64, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE
    assert lib.hot_linear_backward_gw(c, fake, None, 64, 64, 64, fake, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_compress_activation(c, fake, 40, 64, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_compress_activation(c, fake, 64, 64, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE
    assert lib.hot_compress_activation(c, None, 64, 64, fake, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_linear_backward(c, fake, fake, None, 64, 64, 64, 1, fake, fake, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_linear_backward(c, fake, fake, fake, 72, 64, 64, 1, fake, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward(c, fake, fake, fake, 64, 72, 64, 1, fake, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward(c, fake, fake, fake, 64, 64, 64, 1, fake, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE
    assert lib.hot_quantize_weight(c, fake, 72, 64, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_quantize_weight(c, fake, 64, 64, None, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_quantize_weight(c, fake, 64, 64, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE
    assert lib.hot_linear_backward_gx_cached(c, fake, fake, 64, 72, 64, 1, fake, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_linear_backward_gx_cached(c, fake, fake, 64, 64, 64, 1, fake, fake, 100, None) == hot.HOT_ERR_WORKSPACE
    assert lib.hot_linear_backward_gx_cached(c, fake, fake, 64, 64, 64, 3, fake, fake, big, None) == hot.HOT_ERR_ARG
    ch = C.c_int(0)
    assert lib.hot_select_quantizer(c, fake, 64, 64, None, None, None, fake, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_select_quantizer(c, fake, 64, 70, C.byref(ch), None, None, fake, big, None) == hot.HOT_ERR_SHAPE
    assert lib.hot_select_quantizer(c, fake, 64, 64, C.byref(ch), None, None, fake, 10, None) == hot.HOT_ERR_WORKSPACE
    assert hot.status_string(hot.HOT_ERR_WORKSPACE) == "workspace too small"


def test_cached_gx_workspace_covers_the_split_k_scratch():
    """A g_x GEMM with few output tiles splits K and hands partial sums over through scratch
    that follows the g_y codes (L=512, O=I=4096: 128 tiles of 128x128 in 4 slices, 25 MB of images).
    The cached call's workspace is smaller than the uncached one by the weight rows only; a
    workspace that ends with the g_y codes is refused before any launch."""
    lib, cfg = hot.lib(), hot.Config()
    c = C.byref(cfg.c())
    fake = C.c_void_p(4096)
    L, O, I = 512, 4096, 4096
    pitch = O // 2
    codes_end = hot.HOT_WS_PREFIX_BYTES + L * 4 + L * pitch
    full, cached = hot.hot_workspace_bytes(cfg, L, O, I), hot.hot_gx_cached_workspace_bytes(cfg, L, O, I)
    scratch = 128 * 7 * 128 * 128 * 4       # sized for the deepest split a forced mode may ask for
    assert cached == codes_end + scratch
    assert full >= cached + I * pitch
    for too_small in (codes_end, codes_end + 128 * 3 * 128 * 128 * 4, cached - 1):
        assert lib.hot_linear_backward_gx_cached(c, fake, fake, L, O, I, 1, fake, fake, too_small, None) \
            == hot.HOT_ERR_WORKSPACE
    # many output tiles: no split, no scratch, the workspace ends with the g_y codes
    L = 65536
    assert hot.hot_gx_cached_workspace_bytes(cfg, L, O, I) == hot.HOT_WS_PREFIX_BYTES + L * 4 + L * pitch
    assert hot.hot_gx_cached_workspace_bytes(cfg, 64, 72, 64) == 0


def test_workspace_must_be_256_byte_aligned():
    lib, cfg = hot.lib(), hot.Config()
    c = C.byref(cfg.c())
    fake, odd = C.c_void_p(4096), C.c_void_p(4096 + 128)
    big = 1 << 40
    assert lib.hot_linear_backward_gx(c, fake, fake, 64, 64, 64, 1, fake, odd, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_linear_backward_gw(c, fake, fake, 64, 64, 64, fake, odd, big, None) == hot.HOT_ERR_ARG
    assert lib.hot_compress_activation(c, fake, 64, 64, fake, odd, big, None) == hot.HOT_ERR_ARG


def test_lp_l1_rows_match_the_oracles_list():
    """Host-only helper: the library derives the list from the Kronecker factors of H_n, the
    oracle counts sign changes on the explicit matrix; every (n, r) must agree."""
    import ctypes
    import oracle
    for n in (16, 32, 64):
        for r in range(1, n + 1):
            assert hot.hot_lowpass_l1_rows(n, r) == oracle.lowpass_l1_index(n, r).tolist()
    buf = (ctypes.c_int32 * 8)()
    assert hot.lib().hot_lowpass_l1_rows(16, 8, None) == hot.HOT_ERR_ARG
    assert hot.lib().hot_lowpass_l1_rows(24, 8, buf) == hot.HOT_ERR_ARG
    assert hot.lib().hot_lowpass_l1_rows(16, 17, buf) == hot.HOT_ERR_ARG
    # the list is a valid hot_config.keep_idx
    cfg = hot.Config(block=16, keep=8, keep_idx=hot.hot_lowpass_l1_rows(16, 8))
    assert hot.hot_act_buffer_bytes(cfg, 512, 768) == 256 + 512 * 768 // 2


def test_binding_refuses_host_tensors():
    import torch
    cfg = hot.Config()
    x = torch.zeros(64, 64)
    with pytest.raises(ValueError):
        hot.hot_compress_activation(cfg, x, torch.zeros(10, dtype=torch.uint8), torch.zeros(10, dtype=torch.uint8))
