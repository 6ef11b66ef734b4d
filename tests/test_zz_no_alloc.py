"""The allocation-free g_x entry point against hot_linear_backward_gx, through the C ABI.

hot_linear_backward_gx_noalloc runs the same kernels with the library's built-in scratch
array instead of a caller's workspace, so its g_x must be the same bits; the array keeps the
previous call's contents, so a second, smaller call right after a larger one must be as exact
as the first."""
import ctypes as C
import sys

import pytest
import torch

import hot_inputs

pytestmark = pytest.mark.gpu


def _case(hot, L, O, I, n, bits, per_token, seed):
    print(f"[noalloc] L={L} O={O} I={I} n={n} bits={bits} token={per_token}", flush=True)
    sys.stdout.flush()
    name = f"na{L}x{O}x{I}"
    w = hot_inputs.make_w(O, I, seed, name).cuda()
    gy = hot_inputs.make_gy("tok_outlier", L, O, seed, name).cuda()
    cfg = hot.Config(block=n, keep=n // 2, gx_bits=bits)
    q = hot.HOT_Q_PER_TOKEN if per_token else hot.HOT_Q_PER_TENSOR
    want = torch.empty((L, I), device="cuda")
    got = torch.full((L, I), float("nan"), device="cuda")
    ws = hot.alloc_workspace(cfg, L, O, I)
    lib, c = hot.lib(), cfg.c()
    stream = torch.cuda.current_stream().cuda_stream or None
    st = lib.hot_linear_backward_gx(C.byref(c), gy.data_ptr(), w.data_ptr(), L, O, I, q, want.data_ptr(),
                                    ws.data_ptr(), ws.numel(), stream)
    assert st == hot.HOT_OK, hot.status_string(st)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = lib.hot_linear_backward_gx_noalloc(C.byref(c), gy.data_ptr(), w.data_ptr(), L, O, I, q, got.data_ptr(), stream)
    assert st == hot.HOT_OK, hot.status_string(st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(got, want), f"g_x differs from hot_linear_backward_gx at L={L} O={O} I={I}"


def test_noalloc_gx_equals_workspace_gx_on_two_calls_in_a_row():
    import paper_2503_21261_amd as hot
    # a K-splitting GEMM (few tiles, long K), the combined weight / g_y-row launch and the
    # single-pass weight exchange all keep state in the scratch; then a smaller input, a
    # different block size and quantiser, on the same (now dirty) array
    # first the largest shape the array is documented to hold (ViT-B fc1, 59.5 MB of scratch)
    _case(hot, 12608, 3072, 768, 32, 4, True, seed=80)
    _case(hot, 1024, 3072, 768, 32, 4, True, seed=81)
    _case(hot, 264, 448, 136, 16, 4, False, seed=82)
    _case(hot, 130, 2048, 200, 64, 8, True, seed=83)
    _case(hot, 16, 16, 4, 16, 4, True, seed=84)


def test_noalloc_gx_rejects_shapes_beyond_its_scratch_before_any_launch():
    import paper_2503_21261_amd as hot
    cfg = hot.Config()
    c = cfg.c()
    L, O, I = 50432, 3072, 768          # packed g_y codes alone are 77 MB
    assert hot.hot_workspace_bytes(cfg, L, O, I) > hot.HOT_NOALLOC_SCRATCH_BYTES
    fake = C.c_void_p(4096)             # never dereferenced: the call fails its host checks
    st = hot.lib().hot_linear_backward_gx_noalloc(C.byref(c), fake, fake, L, O, I, 1, fake, None)
    assert st == hot.HOT_ERR_SCRATCH_LIMIT
    assert "scratch" in hot.status_string(st)
    assert hot.lib().hot_linear_backward_gx_noalloc(C.byref(c), fake, fake, 64, 72, 64, 1, fake, None) == hot.HOT_ERR_SHAPE
    assert hot.lib().hot_linear_backward_gx_noalloc(C.byref(c), None, fake, 64, 64, 64, 1, fake, None) == hot.HOT_ERR_ARG
