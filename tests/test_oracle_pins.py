"""Pins for the CPU oracle: each test ties it to something other than itself.

The oracle (oracle/dconv_oracle.c) is the definition of the convolution sum
(paper Fig. 3a; Sec. 3 for the one-channel case).  The checks below are
chosen so that a dropped term, a flipped filter, swapped (i, j) or (y, x)
indices, mixed-up channels/filters or a wrong output size each break at
least one of them.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _parse_golden(path):
    blocks, cur = {}, None
    for line in path.read_text().splitlines():
        s = line.strip()
        if not s or s.startswith("#"):
            continue
        if s in ("in", "filt", "out", "mag"):
            cur = s
            blocks[cur] = []
        else:
            blocks[cur].extend(float(t) for t in s.split())
    return blocks


def test_hand_worked_example(golden_dir):
    b = _parse_golden(golden_dir / "hand_example_c2_k2.txt")
    x = np.array(b["in"], np.float32).reshape(1, 2, 3, 3)
    f = np.array(b["filt"], np.float32).reshape(2, 2, 2, 2)
    acc, mag, _ = oracle.general(x, f)
    assert acc.shape == (1, 2, 2, 2)
    np.testing.assert_array_equal(acc.ravel(), np.array(b["out"]))
    np.testing.assert_array_equal(mag.ravel(), np.array(b["mag"]))


@pytest.mark.parametrize("a,b_,c0", [(0, 0, 0), (1, 1, 1), (0, 2, 1), (2, 0, 0), (2, 1, 2)])
def test_delta_filter_selects_shifted_input(a, b_, c0):
    # A filter that is 1 at tap (a, b_) of channel c0 must reproduce the input
    # window shifted by (a, b_), bit for bit: fixes orientation and index order.
    N, C, H, W, K, F = 2, 3, 9, 11, 2, 3
    x, _ = wl.random_case(1, N, C, H, W, K, F)
    f = np.zeros((K, C, F, F), np.float32)
    f[0, c0, a, b_] = 1.0
    f[1, (c0 + 1) % C, F - 1 - a, F - 1 - b_] = 1.0
    acc, mag, o32, _ = oracle.general(x, f, want32=True)
    Ho, Wo = H - F + 1, W - F + 1
    np.testing.assert_array_equal(o32[:, 0], x[:, c0, a:a + Ho, b_:b_ + Wo])
    np.testing.assert_array_equal(
        o32[:, 1], x[:, (c0 + 1) % C, F - 1 - a:F - 1 - a + Ho, F - 1 - b_:F - 1 - b_ + Wo])
    np.testing.assert_array_equal(mag[:, 0], np.abs(x[:, c0, a:a + Ho, b_:b_ + Wo]).astype(np.float64))


def test_box_filter_matches_summed_area_table():
    # All-ones filter: each output is a window sum, obtained here from an fp64
    # integral image -- a different algorithm from the nested loops.
    N, C, H, W, K, F = 2, 3, 17, 23, 2, 5
    x, _ = wl.random_case(2, N, C, H, W, K, F)
    f = np.ones((K, C, F, F), np.float32)
    acc, _, _ = oracle.general(x, f)
    sat = np.zeros((N, C, H + 1, W + 1), np.float64)
    sat[:, :, 1:, 1:] = np.cumsum(np.cumsum(x.astype(np.float64), axis=2), axis=3)
    Ho, Wo = H - F + 1, W - F + 1
    win = (sat[:, :, F:F + Ho, F:F + Wo] - sat[:, :, 0:Ho, F:F + Wo]
           - sat[:, :, F:F + Ho, 0:Wo] + sat[:, :, 0:Ho, 0:Wo]).sum(axis=1)
    for k in range(K):
        np.testing.assert_allclose(acc[:, k], win, rtol=0, atol=1e-11)


@pytest.mark.parametrize("shape", [(2, 3, 10, 13, 4, 3), (1, 1, 12, 9, 3, 5), (3, 5, 8, 8, 2, 1),
                                   (1, 4, 7, 6, 5, 2), (2, 2, 11, 11, 3, 11)])
def test_matches_torch_conv2d_float64(shape):
    # torch's CPU conv2d in float64 is an independent library implementation of
    # the same cross-correlation.
    N, C, H, W, K, F = shape
    x, f = wl.random_case(3, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(f).double())
    np.testing.assert_allclose(acc, ref.numpy(), rtol=0, atol=1e-12 * max(1.0, mag.max()))
    refmag = torch.nn.functional.conv2d(torch.from_numpy(x).double().abs(),
                                        torch.from_numpy(f).double().abs())
    np.testing.assert_allclose(mag, refmag.numpy(), rtol=1e-13, atol=0)


def test_exact_integer_inputs_match_int64_sliding_windows():
    # Integer-valued inputs: the answer is an exact integer; compute it with
    # int64 sliding windows + einsum and demand equality.
    N, C, H, W, K, F = 2, 4, 12, 15, 3, 3
    x, f = wl.integer_case(4, N, C, H, W, K, F)
    acc, mag, o32, _ = oracle.general(x, f, want32=True)
    xi, fi = x.astype(np.int64), f.astype(np.int64)
    win = np.lib.stride_tricks.sliding_window_view(xi, (F, F), axis=(2, 3))  # N C Ho Wo F F
    ref = np.einsum("ncyxij,kcij->nkyx", win, fi)
    np.testing.assert_array_equal(acc, ref.astype(np.float64))
    np.testing.assert_array_equal(o32, ref.astype(np.float32))
    refmag = np.einsum("ncyxij,kcij->nkyx", np.abs(win), np.abs(fi))
    np.testing.assert_array_equal(mag, refmag.astype(np.float64))


def test_linearity_in_input_and_filter():
    N, C, H, W, K, F = 1, 3, 10, 12, 2, 3
    x1, f1 = wl.random_case(5, N, C, H, W, K, F)
    x2, f2 = wl.random_case(6, N, C, H, W, K, F)
    # power-of-two coefficients keep the float32 combinations exact enough to
    # be formed in float32 without rounding ambiguity
    xa = (np.float32(0.5) * x1 + np.float32(2.0) * x2).astype(np.float32)
    a1, _, _ = oracle.general(x1, f1)
    a2, _, _ = oracle.general(x2, f1)
    aa, _, _ = oracle.general(xa, f1)
    comb = 0.5 * a1 + 2.0 * a2
    exact_xa = 0.5 * x1.astype(np.float64) + 2.0 * x2.astype(np.float64)
    # xa is rounded once to float32; allow for that rounding only
    tol = np.abs(exact_xa - xa).max() * np.abs(f1).sum() + 1e-12
    np.testing.assert_allclose(aa, comb, rtol=0, atol=tol)
    fa = (np.float32(0.25) * f1 + np.float32(4.0) * f2).astype(np.float32)
    b1, _, _ = oracle.general(x1, f1)
    b2, _, _ = oracle.general(x1, f2)
    ba, _, _ = oracle.general(x1, fa)
    exact_fa = 0.25 * f1.astype(np.float64) + 4.0 * f2.astype(np.float64)
    tol = np.abs(exact_fa - fa).max() * C * F * F * np.abs(x1).max() + 1e-12
    np.testing.assert_allclose(ba, 0.25 * b1 + 4.0 * b2, rtol=0, atol=tol)


def test_1x1_filter_is_a_channel_matmul():
    N, C, H, W, K, F = 2, 6, 5, 7, 4, 1
    x, f = wl.random_case(7, N, C, H, W, K, F)
    acc, _, _ = oracle.general(x, f)
    ref = torch.matmul(torch.from_numpy(f[:, :, 0, 0]).double(),
                       torch.from_numpy(x).double().reshape(N, C, H * W)).reshape(N, K, H, W)
    np.testing.assert_allclose(acc, ref.numpy(), rtol=0, atol=1e-13)


def test_full_size_filter_is_a_dot_product():
    N, C, H, W, K, F = 2, 3, 6, 6, 2, 6
    x, f = wl.random_case(8, N, C, H, W, K, F)
    acc, _, _ = oracle.general(x, f)
    assert acc.shape == (N, K, 1, 1)
    ref = x.astype(np.float64).reshape(N, -1) @ f.astype(np.float64).reshape(K, -1).T
    np.testing.assert_allclose(acc[:, :, 0, 0], ref, rtol=0, atol=1e-13)


def test_separable_filter_equals_row_then_column_pass():
    H, W, F = 14, 16, 5
    rng = np.random.default_rng(99)
    img = rng.standard_normal((H, W)).astype(np.float32)
    u = rng.integers(-3, 4, F).astype(np.float32)     # vertical taps
    v = rng.integers(-3, 4, F).astype(np.float32)     # horizontal taps
    f = np.outer(u, v).astype(np.float32)[None]       # filt[0][i][j] = u[i] v[j], exact
    acc, _, _ = oracle.single_channel(img, f)
    d = img.astype(np.float64)
    rows = sum(v[j].astype(np.float64) * d[:, j:j + W - F + 1] for j in range(F))
    ref = sum(u[i].astype(np.float64) * rows[i:i + H - F + 1, :] for i in range(F))
    np.testing.assert_allclose(acc[0], ref, rtol=0, atol=1e-12)


def test_single_channel_equals_general_with_one_image_one_channel():
    H, W, K, F = 19, 21, 5, 3
    x, f = wl.random_case(9, 1, 1, H, W, K, F)
    a1, m1, _ = oracle.single_channel(x[0, 0], f[:, 0])
    a2, m2, _ = oracle.general(x, f)
    np.testing.assert_array_equal(a1, a2[0])
    np.testing.assert_array_equal(m1, m2[0])


def test_translation_of_input_translates_output():
    N, C, H, W, K, F = 1, 2, 16, 18, 2, 3
    x, f = wl.random_case(10, N, C, H, W, K, F)
    dy, dx = 2, 3
    acc, _, _ = oracle.general(x, f)
    acc_s, _, _ = oracle.general(np.ascontiguousarray(x[:, :, dy:, dx:]), f)
    np.testing.assert_array_equal(acc_s, acc[:, :, dy:, dx:])


def test_permutations_of_batch_filters_and_channels():
    N, C, H, W, K, F = 3, 4, 9, 9, 5, 3
    x, f = wl.random_case(11, N, C, H, W, K, F)
    acc, _, _ = oracle.general(x, f)
    pn, pk, pc = np.array([2, 0, 1]), np.array([4, 2, 0, 1, 3]), np.array([3, 1, 0, 2])
    a, _, _ = oracle.general(np.ascontiguousarray(x[pn]), f)
    np.testing.assert_array_equal(a, acc[pn])
    a, _, _ = oracle.general(x, np.ascontiguousarray(f[pk]))
    np.testing.assert_array_equal(a, acc[:, pk])
    a, _, _ = oracle.general(np.ascontiguousarray(x[:, pc]), np.ascontiguousarray(f[:, pc]))
    np.testing.assert_allclose(a, acc, rtol=0, atol=1e-13)


def test_sampled_entry_agrees_with_whole_output_and_rectangular_shapes():
    N, C, H, W, K, F = 2, 3, 9, 14, 4, 3          # H != W on purpose
    x, f = wl.random_case(12, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    idx = wl.sample_indices(12, acc.size, 64)
    a, m = oracle.general_at(x, f, idx)
    np.testing.assert_array_equal(a, acc.ravel()[idx])
    np.testing.assert_array_equal(m, mag.ravel()[idx])


def test_thread_count_does_not_change_any_bit():
    N, C, H, W, K, F = 2, 3, 12, 12, 3, 3
    x, f = wl.random_case(13, N, C, H, W, K, F)
    a1, m1, t1 = oracle.general(x, f, threads=1)
    a4, m4, t4 = oracle.general(x, f, threads=4)
    assert t1 == 1 and t4 == 4
    np.testing.assert_array_equal(a1, a4)
    np.testing.assert_array_equal(m1, m4)


def test_oracle_rejects_bad_shapes():
    x = np.zeros((1, 1, 4, 4), np.float32)
    f = np.zeros((1, 1, 5, 5), np.float32)
    with pytest.raises(ValueError):
        oracle.general(x, f)
    with pytest.raises(ValueError):
        oracle.general(x, np.zeros((1, 2, 3, 3), np.float32))


def test_first_config_whole_output_against_torch():
    # The small single-channel benchmark case in full (about 18 MFLOP).
    w = wl.S1
    img, f = wl.make_inputs(w)
    acc, mag, _ = oracle.single_channel(img, f)
    assert acc.shape == w.out_shape()
    ref = torch.nn.functional.conv2d(torch.from_numpy(img).double()[None, None],
                                     torch.from_numpy(f).double()[:, None])[0]
    np.testing.assert_allclose(acc, ref.numpy(), rtol=0, atol=1e-13)
    assert mag.min() >= 0 and np.all(np.abs(acc) <= mag + 1e-15)
