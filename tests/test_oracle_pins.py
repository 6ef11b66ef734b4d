"""Pins for the CPU oracle: every check compares it with something that is not
the oracle itself - an explicit matrix product built with numpy's own kron and
matmul, a closed form, a bound the definition implies, or brute force on tiny
inputs.  A dropped term, wrong sign, wrong index or transposed operand in the
oracle fails at least one of these."""

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(1234)


def H_ref(n):
    """Sec. 3.1 Eq. 2, unnormalised, from numpy's Kronecker product."""
    H1 = np.array([[1, 1], [1, -1]], dtype=np.int64)
    H = np.array([[1]], dtype=np.int64)
    while H.shape[0] < n:
        H = np.kron(H1, H)
    return H


def blockdiag(H, blocks):
    return np.kron(np.eye(blocks, dtype=np.int64), H)


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_hadamard_matrix_recurrence_and_orthogonality(n):
    H = oracle.hadamard(n).astype(np.int64)
    assert np.array_equal(H, H_ref(n))
    assert np.array_equal(H @ H.T, n * np.eye(n, dtype=np.int64))  # Eq. 3: H^T H = n I
    assert np.array_equal(H, H.T)


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_fwht_equals_explicit_product_exactly_on_integers(n):
    H = H_ref(n)
    for _ in range(20):
        v = RNG.integers(-1000, 1000, size=n)
        out = oracle.fwht(v.astype(np.float32))
        assert np.array_equal(out.astype(np.int64), H @ v)
        # involution: H_u H_u v = n v
        assert np.array_equal(oracle.fwht(out).astype(np.int64), n * v)
    # unit vectors pick out the columns of H: wrong pairing or sign shows here
    for k in range(n):
        e = np.zeros(n, dtype=np.float32)
        e[k] = 1
        assert np.array_equal(oracle.fwht(e).astype(np.int64), H[:, k])


@pytest.mark.parametrize("n", [16, 32, 64])
def test_fwht_float_close_to_double_product(n):
    v = RNG.standard_normal(n).astype(np.float32)
    ref = H_ref(n).astype(np.float64) @ v.astype(np.float64)
    out = oracle.fwht(v)
    assert np.max(np.abs(out - ref)) <= 8 * np.finfo(np.float32).eps * np.sum(np.abs(v))


def test_fwht_rounding_order_is_the_butterfly_tree():
    """fp32 result equals the stage-by-stage butterfly evaluated in numpy fp32
    (h = 1, 2, 4, ...), which is a specific summation tree; a different stage
    order rounds differently on these inputs."""
    n = 16
    diff_seen = False
    for _ in range(50):
        v = (RNG.standard_normal(n) * 10.0 ** RNG.integers(-3, 4, size=n)).astype(np.float32)
        a = v.copy()
        h = 1
        while h < n:
            a = a.reshape(-1, 2, h)
            a = np.stack([a[:, 0, :] + a[:, 1, :], a[:, 0, :] - a[:, 1, :]], axis=1).reshape(-1)
            h *= 2
        assert np.array_equal(oracle.fwht(v), a.astype(np.float32))
        b = v.copy()  # reversed stage order: same mathematics, different rounding
        h = n // 2
        while h >= 1:
            b = b.reshape(-1, 2, h)
            b = np.stack([b[:, 0, :] + b[:, 1, :], b[:, 0, :] - b[:, 1, :]], axis=1).reshape(-1)
            h //= 2
        diff_seen |= not np.array_equal(a, b)
    assert diff_seen


@pytest.mark.parametrize("n", [16, 32, 64])
def test_transform_rows_and_hla_equal_block_diagonal_products(n):
    L, O, I = 2 * n, 3 * n, 5
    g = RNG.integers(-50, 50, size=(L, O))
    w = RNG.integers(-50, 50, size=(O, I))
    H = H_ref(n)
    T = oracle.transform_rows(g.astype(np.float32), n)
    assert np.array_equal(T.astype(np.int64), g @ blockdiag(H, O // n).T)  # g_y H^T
    ident = np.arange(n)
    U = oracle.hla(w.astype(np.float32), n, n, ident)
    assert np.array_equal(U.astype(np.int64), blockdiag(H, O // n) @ w)    # H w
    # Eq. 3 with Q removed: (g H^T)(H w) / n = g w exactly on integers
    assert np.array_equal(T.astype(np.int64) @ U.astype(np.int64), n * (g @ w))
    # reduced rank: rows keep[j] of every block, output row b*r + j
    r = n // 4
    keep = RNG.permutation(n)[:r]
    x = RNG.integers(-50, 50, size=(L, I))
    xh = oracle.hla(x.astype(np.float32), n, r, keep)
    full = (blockdiag(H, L // n) @ x).reshape(L // n, n, I)
    assert np.array_equal(xh.astype(np.int64), full[:, keep, :].reshape(L // n * r, I))


def _gray_inverse(g):
    b = 0
    while g:
        b ^= g
        g >>= 1
    return b


def _bitrev(k, bits):
    return int(format(k, f"0{bits}b")[::-1], 2)


@pytest.mark.parametrize("n", [4, 16, 32, 64])
def test_sequency_brute_force_matches_closed_form_and_lowpass_set(n):
    bits = n.bit_length() - 1
    H = H_ref(n)
    seq_np = [(np.diff(H[k]) != 0).sum() for k in range(n)]
    for k in range(n):
        assert oracle.sequency(n, k) == seq_np[k] == _gray_inverse(_bitrev(k, bits))
    assert sorted(seq_np) == list(range(n))
    for r in (1, n // 4, n // 2, n):
        idx = oracle.lowpass_index(n, r)
        assert [seq_np[k] for k in idx] == list(range(r))
    # the n/2 lowest-sequency rows are the even natural indices
    assert sorted(oracle.lowpass_index(n, n // 2)) == list(range(0, n, 2))


@pytest.mark.parametrize("n,r", [(16, 8), (16, 4), (32, 16), (64, 32), (64, 8)])
def test_lowpass_hla_is_projection_on_run_means(n, r):
    """With the r = n/2^k lowest-sequency rows kept, H_hat^T H_hat / n projects
    onto functions constant on runs of m = n/r tokens, so the unquantised HLA
    weight gradient is  sum_runs m * mean(g_y)^T mean(x)  - no WHT involved."""
    L, O, I = 4 * n, 6, 5
    g = RNG.standard_normal((L, O)).astype(np.float32)
    x = RNG.standard_normal((L, I)).astype(np.float32)
    keep = oracle.lowpass_index(n, r)
    gh = oracle.hla(g, n, r, keep).astype(np.float64)
    xh = oracle.hla(x, n, r, keep).astype(np.float64)
    m = n // r
    gm = g.astype(np.float64).reshape(L // m, m, O).mean(axis=1)
    xm = x.astype(np.float64).reshape(L // m, m, I).mean(axis=1)
    np.testing.assert_allclose(gh.T @ xh / n, m * gm.T @ xm, rtol=0, atol=1e-4)


@pytest.mark.parametrize("n", [16, 32])
def test_full_rank_hla_reproduces_exact_weight_gradient(n):
    L, O, I = 8 * n, 24, 40
    g = RNG.standard_normal((L, O)).astype(np.float32)
    x = RNG.standard_normal((L, I)).astype(np.float32)
    ident = np.arange(n)
    gh = oracle.hla(g, n, n, ident).astype(np.float64)
    xh = oracle.hla(x, n, n, ident).astype(np.float64)
    exact = g.astype(np.float64).T @ x.astype(np.float64)
    np.testing.assert_allclose(gh.T @ xh / n, exact, rtol=0, atol=1e-3)
    # and through the whole INT8 g_w path the error is a fraction of a percent
    codes, sx = oracle.compress_activation(x, n, n, keep=ident, rounding=oracle.NEAREST_EVEN)
    out = oracle.backward_gw(g, codes, sx, n, n, keep=ident, rounding=oracle.NEAREST_EVEN)
    rel = np.linalg.norm(out["g_w"] - exact) / np.linalg.norm(exact)
    assert rel < 0.02, rel
    assert out["overflow"] == 0


def _grid(n):
    return (4, 4) if n == 16 else ((4, 8) if n == 32 else (8, 8))


@pytest.mark.parametrize("n", [16, 32, 64])
def test_lp_l1_rows_are_the_lowest_two_dimensional_sequencies(n):
    """The LP_L1 list (Supp. B) as read by the oracle, pinned by what any reading of it must
    satisfy and by a second construction: rows of H_n as images on the token grid, built here
    from numpy's Kronecker product of the two 1-D factors rather than from the oracle's matrix."""
    gh, gw = _grid(n)
    Hh, Hw = H_ref(gh), H_ref(gw)
    assert np.array_equal(np.kron(Hh, Hw), H_ref(n))            # the grid reading of a block
    seq_h = [(np.diff(Hh[a]) != 0).sum() for a in range(gh)]
    seq_w = [(np.diff(Hw[b]) != 0).sum() for b in range(gw)]
    l1 = np.array([seq_h[k // gw] + seq_w[k % gw] for k in range(n)])
    full = oracle.lowpass_l1_index(n, n)
    assert sorted(full.tolist()) == list(range(n))               # every row once: full rank
    assert full[0] == 0                                          # the constant vector comes first
    assert np.all(np.diff(l1[full]) >= 0)                        # non-decreasing L1 norm of the 2-D sequency
    for r in range(1, n + 1):
        idx = oracle.lowpass_l1_index(n, r)
        assert idx.tolist() == full[:r].tolist()                 # prefixes of one order
        dropped = np.setdiff1d(np.arange(n), idx)
        assert dropped.size == 0 or l1[idx].max() <= l1[dropped].min()
    if gh == gw:
        # turning the grid over (vertical <-> horizontal) maps row a*g + b to b*g + a; whenever the
        # kept rows end on a boundary of the tie-break's own classes the set does not change
        key = [(l1[k], max(seq_h[k // gw], seq_w[k % gw])) for k in range(n)]
        for r in range(1, n + 1):
            if r == n or key[full[r - 1]] != key[full[r]]:
                idx = oracle.lowpass_l1_index(n, r)
                flipped = sorted((k % gw) * gw + k // gw for k in idx)
                assert flipped == sorted(idx.tolist()), r
        assert any(key[full[r - 1]] != key[full[r]] for r in (n // 2,))   # the paper's 8 of 16 is such an r


def test_lp_l1_sixteen_tokens_keep_eight_is_the_two_by_two_corner_plus_two_edges():
    """n = 16, r = 8: sequency pairs (vertical, horizontal) with sum <= 2, and of the four with
    sum 3 the two that are not on an axis: (1,2) and (2,1)."""
    Hh = H_ref(4)
    seq = [(np.diff(Hh[a]) != 0).sum() for a in range(4)]
    pairs = sorted((seq[k // 4], seq[k % 4]) for k in oracle.lowpass_l1_index(16, 8))
    assert pairs == sorted([(0, 0), (0, 1), (1, 0), (1, 1), (0, 2), (2, 0), (1, 2), (2, 1)])


@pytest.mark.parametrize("n", [16, 64])
def test_lp_l1_full_rank_reproduces_exact_weight_gradient_and_low_rank_is_a_two_d_low_pass(n):
    L, O, I = 4 * n, 6, 5
    g = RNG.standard_normal((L, O)).astype(np.float32)
    x = RNG.standard_normal((L, I)).astype(np.float32)
    keep = oracle.lowpass_l1_index(n, n)
    gh_, xh_ = oracle.hla(g, n, n, keep).astype(np.float64), oracle.hla(x, n, n, keep).astype(np.float64)
    np.testing.assert_allclose(gh_.T @ xh_ / n, g.astype(np.float64).T @ x.astype(np.float64), rtol=0, atol=1e-3)
    # r = 4: the rows with both sequencies <= 1 span the functions that are constant on the four
    # quadrants of the grid, so the unquantised result is the sum over quadrants of
    # (tokens per quadrant) * mean(g_y)^T mean(x): no transform involved
    gdim = _grid(n)[0]
    keep4 = oracle.lowpass_l1_index(n, 4)
    g4, x4 = oracle.hla(g, n, 4, keep4).astype(np.float64), oracle.hla(x, n, 4, keep4).astype(np.float64)
    def quadrant_means(t):
        t = t.astype(np.float64).reshape(L // n, 2, gdim // 2, 2, gdim // 2, t.shape[1])
        return t.mean(axis=(2, 4)).reshape(L // n * 4, -1)
    np.testing.assert_allclose(g4.T @ x4 / n, (n // 4) * quadrant_means(g).T @ quadrant_means(x), rtol=0, atol=1e-4)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("per_token", [False, True])
def test_quantizer_bounds_range_and_scales(bits, per_token):
    qmax = 2 ** (bits - 1) - 1
    t = (RNG.standard_normal((37, 96)) * np.exp(RNG.standard_normal((37, 1)))).astype(np.float32)
    t[5, :] = 0.0  # an all-zero token
    for rounding, bound in ((oracle.NEAREST_EVEN, 0.5), (oracle.PSEUDO_STOCHASTIC, 1.0)):
        q, s = oracle.quantize(t, bits, per_token, rounding)
        assert q.min() >= -qmax and q.max() <= qmax
        amax = np.abs(t).max(axis=1) if per_token else np.abs(t).max(keepdims=True).reshape(1)
        np.testing.assert_array_equal(s, (amax / np.float32(qmax)).astype(np.float32))
        srow = s[:, None] if per_token else s[0]
        err = np.abs(q.astype(np.float64) * srow - t)
        assert np.all(err <= bound * srow * (1 + 1e-5) + 1e-30)
        if per_token:
            assert np.all(q[5] == 0) and s[5] == 0.0
            hit = np.abs(q).max(axis=1)
            assert np.all(np.delete(hit, 5) == qmax)  # the abs-max element maps to +-qmax
        else:
            assert np.abs(q).max() == qmax
    if bits == 4:
        q, s = oracle.quantize(np.zeros((3, 16), np.float32), bits, per_token, oracle.PSEUDO_STOCHASTIC)
        assert not q.any() and not s.any()


def test_nearest_even_is_rint_and_ties_go_to_even():
    # amax = 7 -> inv = 1 exactly, so codes are the rounded values themselves
    t = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, 3.51, -6.5, 6.5]], np.float32)
    q, s = oracle.quantize(t, 4, True, oracle.NEAREST_EVEN)
    assert s[0] == 1.0
    assert q[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 3, 4, -6, 6]


def test_pseudo_stochastic_worked_examples():
    """Hand-evaluated cases of the rounding rule (reading of Sec. 5.1): with
    amax = 7 the scaled value equals the input; its low 11 pattern bits / 2048
    are the threshold for the fractional part."""
    ulp2 = np.float32(2.0 ** -22)  # spacing of fp32 in [2, 4)
    cases = [
        (2.5, 3),                      # low bits 0 -> threshold 0, any positive fraction rounds up
        (2.0, 2),                      # exact integers never move
        (-2.0, -2),
        (-2.25, -2),                   # floor -3, frac .75 > 0
        (2.25 + 1023 * ulp2, 2),       # threshold 1023/2048 ~ .4995, frac ~ .2502
        (2.75 + 1023 * ulp2, 3),       # same threshold, frac ~ .7502
        (2.0 + 2047 * ulp2, 2),        # threshold .9995, frac ~ .00049
        (3.0 - ulp2, 3),               # pattern ends in 0x7FF: threshold .9995 < frac .99999976
    ]
    vals = np.array([[7.0] + [c[0] for c in cases]], dtype=np.float32)
    q, s = oracle.quantize(vals, 4, True, oracle.PSEUDO_STOCHASTIC)
    assert s[0] == 1.0
    assert q[0, 1:].tolist() == [c[1] for c in cases]


def test_pseudo_stochastic_rounding_is_unbiased_in_the_mean():
    t = RNG.standard_normal((64, 65536)).astype(np.float32)
    for bits in (4, 8):
        q, s = oracle.quantize(t, bits, False, oracle.PSEUDO_STOCHASTIC)
        err = q.astype(np.float64) * s[0] - t
        n = err.size
        # stochastic rounding: per-element error std <= s/2, so the mean is within a few s/sqrt(n)
        assert abs(err.mean()) < 4 * 0.5 * s[0] / np.sqrt(n)
        # deterministic nearest rounding of the same data is NOT what is being measured:
        # floor would give a mean of -s/2
        assert abs(err.mean()) < 0.01 * s[0]


def test_integer_gemm_brute_force_and_numpy():
    A = RNG.integers(-7, 8, size=(3, 5)).astype(np.int8)
    B = RNG.integers(-7, 8, size=(5, 4)).astype(np.int8)
    acc, bad = oracle.igemm_nn(A, B)
    brute = [[sum(int(A[m, k]) * int(B[k, j]) for k in range(5)) for j in range(4)] for m in range(3)]
    assert acc.tolist() == brute and bad == 0
    At = np.ascontiguousarray(A.T)
    acc_t, _ = oracle.igemm_tn(At, B)
    assert acc_t.tolist() == brute
    A = RNG.integers(-127, 128, size=(33, 257)).astype(np.int8)
    B = RNG.integers(-127, 128, size=(257, 19)).astype(np.int8)
    ref = A.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(oracle.igemm_nn(A, B)[0], ref)
    assert np.array_equal(oracle.igemm_tn(np.ascontiguousarray(A.T), B)[0], ref)
    # accumulators beyond int32 are counted
    A = np.full((1, 140000), 127, np.int8)
    B = np.full((140000, 1), 127, np.int8)
    acc, bad = oracle.igemm_nn(A, B)
    assert acc[0, 0] == 127 * 127 * 140000 and bad == 1


def test_token_scale_factors_out_of_the_product_row():
    """Sec. 4.3: diag(s_g) (Qg Qw) s_w / n equals the product of the dequantised
    operands."""
    n = 16
    g = (RNG.standard_normal((32, 48)) * np.exp(2 * RNG.standard_normal((32, 1)))).astype(np.float32)
    w = (0.02 * RNG.standard_normal((48, 24))).astype(np.float32)
    out = oracle.backward_gx(g, w, n, bits=4, per_token=True)
    deq_g = out["qg"].astype(np.float64) * out["sg"].astype(np.float64)[:, None]
    deq_w = out["qw"].astype(np.float64) * float(out["sw"][0])
    np.testing.assert_allclose(out["g_x"], deq_g @ deq_w / n, rtol=1e-12, atol=0)
    assert np.array_equal(out["acc"], out["qg"].astype(np.int64) @ out["qw"].astype(np.int64))
    # taps agree with the stage functions
    T = oracle.transform_rows(g, n)
    q, s = oracle.quantize(T, 4, True, oracle.PSEUDO_STOCHASTIC)
    assert np.array_equal(q, out["qg"]) and np.array_equal(s, out["sg"])


@pytest.mark.parametrize("n,bits,tol", [(16, 8, 0.03), (16, 4, 0.45), (32, 8, 0.03), (64, 4, 0.45)])
def test_gx_path_approximates_exact_gradient(n, bits, tol):
    """Eq. 3-4: with Q close to the identity (INT8) the rotated, quantised product
    must be close to g_y w; a transposed operand, a missing 1/n or a wrong scale
    gives an O(1) error.  INT4 stays within the error the 7-level grid implies."""
    L, O, I = 64, 4 * n, 48
    g = RNG.standard_normal((L, O)).astype(np.float32) * 1e-3
    w = (0.02 * RNG.standard_normal((O, I))).astype(np.float32)
    x = RNG.standard_normal((L, I)).astype(np.float32)
    exact_gx, _ = oracle.exact_backward(g, x, w, want_gw=False)
    np.testing.assert_allclose(exact_gx, g.astype(np.float64) @ w.astype(np.float64), rtol=1e-12)
    for per_token in (True, False):
        out = oracle.backward_gx(g, w, n, bits=bits, per_token=per_token)
        rel = np.linalg.norm(out["g_x"] - exact_gx) / np.linalg.norm(exact_gx)
        assert rel < tol, (per_token, rel)


def test_gw_path_with_default_lowpass_approximates_smooth_activations():
    """HLA keeps low sequencies (Sec. 4.2: the sum over L acts as a low-pass
    filter): for token sequences that are constant on runs of n/r tokens the
    rank-r path is exact up to INT8 quantisation."""
    n, r, L, O, I = 16, 8, 256, 24, 40
    g = np.repeat(RNG.standard_normal((L // 2, O)), 2, axis=0).astype(np.float32)
    x = np.repeat(RNG.standard_normal((L // 2, I)), 2, axis=0).astype(np.float32)
    codes, sx = oracle.compress_activation(x, n, r)
    assert codes.shape == (L * r // n, I) and codes.nbytes * 8 == x.nbytes  # 12.5 % (Sec. 5.2.1)
    out = oracle.backward_gw(g, codes, sx, n, r)
    _, exact = oracle.exact_backward(g, x, np.zeros((O, I), np.float32), want_gx=False)
    np.testing.assert_allclose(exact, g.astype(np.float64).T @ x.astype(np.float64), rtol=1e-12)
    rel = np.linalg.norm(out["g_w"] - exact) / np.linalg.norm(exact)
    assert rel < 0.02, rel
    assert np.array_equal(out["acc"], out["qg"].astype(np.int64).T @ codes.astype(np.int64))


def test_select_quantizer_mse_in_original_domain_and_end_points():
    n, L, O = 16, 48, 64
    H = H_ref(n).astype(np.float64)
    B = blockdiag(H, O // n).astype(np.float64)
    g = (RNG.standard_normal((L, O)) * 1e-3).astype(np.float32)
    choice, m_tok, m_ten = oracle.select_quantizer(g, n, bits=4)
    # independent evaluation: dequantise, rotate back with H^T / n, compare with g_y itself
    T = oracle.transform_rows(g, n)
    for per_token, got in ((True, m_tok), (False, m_ten)):
        q, s = oracle.quantize(T, 4, per_token, oracle.PSEUDO_STOCHASTIC)
        deq = q.astype(np.float64) * (s.astype(np.float64)[:, None] if per_token else float(s[0]))
        back = deq @ B / n            # (H_u^T H_u = n I)
        mse = np.mean((back - g.astype(np.float64)) ** 2)
        # the fp32 rotation rounds (~1e-7 relative per element), hence not 1e-12
        np.testing.assert_allclose(got, mse, rtol=1e-6)
    # rows with identical abs-max after rotation: identical codes, no gain -> per-tensor
    row = RNG.standard_normal(O).astype(np.float32)
    same = np.tile(row, (L, 1))
    choice, m_tok, m_ten = oracle.select_quantizer(same, n)
    assert not choice and m_tok == m_ten
    # a few tokens 50x larger: per-tensor wastes the grid on them -> per-token
    out = g.copy()
    out[::12] *= 50
    choice, m_tok, m_ten = oracle.select_quantizer(out, n)
    assert choice and m_tok < 0.5 * m_ten
    # all-zero gradient: nothing to gain
    assert oracle.select_quantizer(np.zeros((L, O), np.float32), n)[0] is False


# ---- bf16 variant of the g_w path ---------------------------------------------------------

def test_bf16_rounding_matches_an_independent_conversion_and_the_tie_rule():
    import torch
    rng = np.random.default_rng(11)
    a = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, 1.0, -1.0, 3.0e38, 1e-40], dtype=np.float32)])
    mine = oracle.bf16_bits(a)
    theirs = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, theirs)
    # exact ties: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> even (1); 1 + 3*2^-8 -> 1 + 2^-6
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8)], dtype=np.float32)
    assert np.array_equal(oracle.bf16_value(oracle.bf16_bits(ties)),
                          np.array([1.0, 1.0 + 2.0 ** -6, -1.0], dtype=np.float32))
    # values already representable are untouched
    exact = np.array([0.5, -2.75, 96.0, 2.0 ** -100], dtype=np.float32)
    assert np.array_equal(oracle.bf16_value(oracle.bf16_bits(exact)), exact)


def test_bf16_gw_is_the_exact_product_of_its_rounded_operands_and_close_to_hla():
    rng = np.random.default_rng(12)
    L, O, I, n, r = 128, 24, 20, 16, 8
    gy = (rng.standard_normal((L, O)) * 1e-3).astype(np.float32)
    x = rng.standard_normal((L, I)).astype(np.float32)
    xb = oracle.compress_activation_bf16(x, n, r)
    out = oracle.backward_gw_bf16(gy, xb, n, r)
    keep = oracle.lowpass_index(n, r)
    gh = oracle.hla(gy, n, r, keep).astype(np.float64)
    xh = oracle.hla(x, n, r, keep).astype(np.float64)
    # brute force over the rounded operands, term by term
    A, B = oracle.bf16_value(out["gh_bits"]).astype(np.float64), oracle.bf16_value(xb).astype(np.float64)
    brute = np.zeros((O, I))
    for k in range(A.shape[0]):
        brute += np.outer(A[k], B[k])
    np.testing.assert_allclose(out["g_w"], brute / n, rtol=1e-12, atol=1e-18)
    # each operand is within 2^-9 relative of the unrounded one, so every term is within
    # ~2^-8 and the result within 2^-8 * sum |terms|
    bound = 2.0 ** -8 * (np.abs(gh).T @ np.abs(xh)) / n + 1e-30
    assert (np.abs(out["g_w"] - gh.T @ xh / n) <= bound).all()


def test_bf16_gw_full_rank_reproduces_the_exact_gradient_for_bf16_exact_inputs():
    """r = n and inputs whose transformed values are exactly representable in bfloat16
    (small integers): the reduced-rank bf16 path is then the exact g_y^T x."""
    rng = np.random.default_rng(13)
    L, O, I, n = 64, 8, 6, 16
    gy = rng.integers(-3, 4, size=(L, O)).astype(np.float32)
    x = rng.integers(-3, 4, size=(L, I)).astype(np.float32)
    keep = np.arange(n, dtype=np.int32)
    xb = oracle.compress_activation_bf16(x, n, n, keep)
    out = oracle.backward_gw_bf16(gy, xb, n, n, keep)
    assert np.array_equal(out["g_w"], gy.astype(np.float64).T @ x.astype(np.float64))


# ---- per-sample tiling -------------------------------------------------------------------

def test_per_sample_tiling_is_the_concatenation_of_independent_samples_and_exact_at_full_rank():
    rng = np.random.default_rng(21)
    B, S, O, I, n, r = 3, 23, 6, 5, 16, 8        # 23 tokens: one full block and one of 7 + 9 zeros
    gy = rng.integers(-4, 5, size=(B * S, O)).astype(np.float32)
    x = rng.integers(-4, 5, size=(B * S, I)).astype(np.float32)
    keep = oracle.lowpass_index(n, r)
    whole = oracle.hla(oracle.pad_samples(x, S, n), n, r, keep)
    Sp = 32
    for b in range(B):      # each sample on its own, padded by hand
        one = np.zeros((Sp, I), dtype=np.float32)
        one[:S] = x[b * S:(b + 1) * S]
        assert np.array_equal(whole[b * (Sp // n) * r:(b + 1) * (Sp // n) * r], oracle.hla(one, n, r, keep))
    # full rank: the zero tokens contribute nothing, the product is the exact gradient
    full = np.arange(n, dtype=np.int32)
    gh = oracle.hla(oracle.pad_samples(gy, S, n), n, n, full).astype(np.float64)
    xh = oracle.hla(oracle.pad_samples(x, S, n), n, n, full).astype(np.float64)
    assert np.array_equal(gh.T @ xh / n, gy.astype(np.float64).T @ x.astype(np.float64))


# ---- values the paper itself prints (fixtures under tests/golden/, each with its citation) ----

def _golden(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    return np.array(rows, dtype=np.float64)


def test_golden_h2_sign_matrix_and_its_transform():
    S = _golden("hadamard_h2.txt")
    assert np.array_equal(oracle.hadamard(4).astype(np.float64), S)
    v = np.array([3.0, -1.0, 4.0, 1.5], dtype=np.float32)
    assert np.array_equal(oracle.fwht(v).astype(np.float64), S @ v.astype(np.float64))
    # one more application of the recurrence, H_3 = H_1 (x) H_2, checked block by block
    H8 = oracle.hadamard(8).astype(np.float64)
    assert np.array_equal(H8[:4, :4], S) and np.array_equal(H8[:4, 4:], S)
    assert np.array_equal(H8[4:, :4], S) and np.array_equal(H8[4:, 4:], -S)


def test_golden_activation_buffer_ratio():
    frac, stored, orig, ratio = _golden("abc_ratio.txt")[0]
    assert frac * stored / orig == ratio
    L, I, n = 512, 96, 16
    r = int(n * frac)
    x = np.random.default_rng(3).standard_normal((L, I)).astype(np.float32)
    codes, _ = oracle.compress_activation(x, n, r)
    assert codes.dtype == np.int8 and codes.nbytes == ratio * x.nbytes
