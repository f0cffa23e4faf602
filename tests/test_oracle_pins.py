"""CPU-only pins of the fp64 oracle against things other than itself.

The oracle is the operator definition of Sec. IV-A (eqs. (dwconv), (dx_def)
read as the adjoint, (dk_def)).  Each test below fixes it to something the
mathematics or a library routine decides: hand-worked values, closed forms,
a scatter-form brute force, fp64 grouped conv1d and its autograd (the paper's
own validation protocol, App. A "Validation Protocol"), finite differences and
the adjoint identity.
"""
import json
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))

TINY = [(1, 1, 5, 3), (2, 3, 7, 4), (1, 2, 4, 6), (2, 2, 9, 1), (1, 3, 3, 8), (3, 1, 16, 5)]


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def all_pads(K):
    return list(range(K))


# ---------------------------------------------------------------- golden, hand-worked
def test_hand_worked_examples(oracle_mod):
    with open(os.path.join(HERE, "golden", "worked_examples.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 3
    for cs in cases:
        L, K, p = cs["L"], cs["K"], cs["pad_left"]
        x = np.array(cs["x"], np.float32).reshape(1, 1, L)
        w = np.array(cs["w"], np.float32).reshape(1, K)
        dy = np.array(cs["dy"], np.float32).reshape(1, 1, L)
        y, _ = oracle_mod.fwd(x, w, p)
        dx, _ = oracle_mod.bwd_input(dy, w, p)
        dw, _ = oracle_mod.bwd_weight(x, dy, K, p)
        assert y.ravel().tolist() == cs["y"], cs["cite"]
        assert dx.ravel().tolist() == cs["dx"], cs["cite"]
        assert dw.ravel().tolist() == cs["dw"], cs["cite"]
        assert float((dy.astype(np.float64) * y).sum()) == cs["inner"]


# ---------------------------------------------------------------- closed forms, forward
@pytest.mark.parametrize("B,C,L,K", [(2, 3, 11, 5), (1, 2, 6, 6), (1, 1, 4, 9)])
def test_fwd_identity_filter_is_shift(oracle_mod, B, C, L, K):
    x = rnd((B, C, L), 1)
    for p in all_pads(K):
        for j0 in range(K):
            w = np.zeros((C, K), np.float32)
            w[:, j0] = 1.0
            y, ya = oracle_mod.fwd(x, w, p)
            exp = np.zeros((B, C, L))
            for t in range(L):
                u = t + j0 - p
                if 0 <= u < L:
                    exp[:, :, t] = x[:, :, u]
            assert np.array_equal(y, exp)
            assert np.array_equal(ya, np.abs(exp))
            if j0 == p:
                assert np.array_equal(y, x.astype(np.float64))


@pytest.mark.parametrize("L,K", [(9, 4), (5, 7), (8, 8)])
def test_fwd_delta_input_lays_reversed_filter(oracle_mod, L, K):
    C = 2
    w = rnd((C, K), 2)
    for p in all_pads(K):
        for t0 in range(L):
            x = np.zeros((1, C, L), np.float32)
            x[0, :, t0] = 1.0
            y, _ = oracle_mod.fwd(x, w, p)
            for t in range(L):
                j = t0 - t + p
                exp = w[:, j].astype(np.float64) if 0 <= j < K else np.zeros(C)
                assert np.array_equal(y[0, :, t], exp)


@pytest.mark.parametrize("B,C,L,K", [(2, 2, 10, 4), (1, 1, 3, 7)])
def test_all_ones_count_taps(oracle_mod, B, C, L, K):
    x = np.ones((B, C, L), np.float32)
    w = np.ones((C, K), np.float32)
    for p in all_pads(K):
        y, ya = oracle_mod.fwd(x, w, p)
        dx, _ = oracle_mod.bwd_input(x, w, p)
        dw, dwa = oracle_mod.bwd_weight(x, x, K, p)
        for t in range(L):
            n_f = sum(1 for j in range(K) if 0 <= t + j - p < L)
            n_b = sum(1 for j in range(K) if 0 <= t - j + p < L)
            assert np.all(y[:, :, t] == n_f) and np.all(ya[:, :, t] == n_f)
            assert np.all(dx[:, :, t] == n_b)
        for j in range(K):
            assert np.all(dw[:, j] == B * max(0, L - abs(j - p)))   # closed form
            assert np.all(dwa[:, j] == B * max(0, L - abs(j - p)))


# ---------------------------------------------------------------- brute force, scatter form
def scatter_forms(x, w, dy, p):
    """Differently-structured evaluation: visit every (input s, tap j) pair once and
    scatter x[s]*w[j] into y[s-j+p]; gradients visit the same pairs."""
    B, C, L = x.shape
    K = w.shape[1]
    y = np.zeros((B, C, L)); dx = np.zeros((B, C, L)); dw = np.zeros((C, K))
    for b in range(B):
        for c in range(C):
            for s in range(L):
                for j in range(K):
                    t = s - j + p
                    if 0 <= t < L:
                        y[b, c, t] += float(x[b, c, s]) * float(w[c, j])
                        dx[b, c, s] += float(dy[b, c, t]) * float(w[c, j])
                        dw[c, j] += float(dy[b, c, t]) * float(x[b, c, s])
    return y, dx, dw


@pytest.mark.parametrize("B,C,L,K", TINY)
def test_against_scatter_brute_force(oracle_mod, B, C, L, K):
    x = rnd((B, C, L), 3); w = rnd((C, K), 4); dy = rnd((B, C, L), 5)
    for p in all_pads(K):
        ys, dxs, dws = scatter_forms(x, w, dy, p)
        y, _ = oracle_mod.fwd(x, w, p)
        dx, _ = oracle_mod.bwd_input(dy, w, p)
        dw, _ = oracle_mod.bwd_weight(x, dy, K, p)
        np.testing.assert_allclose(y, ys, rtol=0, atol=1e-13)
        np.testing.assert_allclose(dx, dxs, rtol=0, atol=1e-13)
        np.testing.assert_allclose(dw, dws, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- library routine: grouped conv1d, fp64
def torch_reference(x, w, dy, p):
    """fp64 grouped conv1d on explicitly padded input, and its autograd."""
    K = w.shape[1]
    xt = torch.from_numpy(x).double().requires_grad_(True)
    wt = torch.from_numpy(w).double().requires_grad_(True)
    xp = torch.nn.functional.pad(xt, (p, K - 1 - p))
    y = torch.nn.functional.conv1d(xp, wt[:, None, :], groups=w.shape[0])
    y.backward(torch.from_numpy(dy).double())
    return y.detach().numpy(), xt.grad.numpy(), wt.grad.numpy()


@pytest.mark.parametrize("B,C,L,K,p", [
    (2, 5, 37, 7, 3), (3, 4, 50, 16, 15), (2, 3, 48, 48, 24), (1, 6, 33, 12, 0),
    (2, 2, 20, 31, 15), (2, 3, 64, 9, 8), (1, 2, 10, 25, 24), (4, 8, 129, 64, 63)])
def test_against_fp64_grouped_conv1d_and_autograd(oracle_mod, B, C, L, K, p):
    x = rnd((B, C, L), 6); w = rnd((C, K), 7); dy = rnd((B, C, L), 8)
    yt, dxt, dwt = torch_reference(x, w, dy, p)
    y, ya = oracle_mod.fwd(x, w, p)
    dx, dxa = oracle_mod.bwd_input(dy, w, p)
    dw, dwa = oracle_mod.bwd_weight(x, dy, K, p)
    assert np.max(np.abs(y - yt) / np.maximum(ya, 1e-300)) < 1e-13
    assert np.max(np.abs(dx - dxt) / np.maximum(dxa, 1e-300)) < 1e-13
    assert np.max(np.abs(dw - dwt) / np.maximum(dwa, 1e-300)) < 1e-13


def test_even_K_paper_convention_pad_both_sides_then_crop(oracle_mod):
    """App. A: for even K the library reference pads K/2 on both sides and the output is
    cropped to L; keeping outputs t = 0..L-1 equals eq. (dwconv) with p = K/2."""
    B, C, L, K = 2, 3, 48, 48
    x = rnd((B, C, L), 9); w = rnd((C, K), 10)
    full = torch.nn.functional.conv1d(torch.from_numpy(x).double(), torch.from_numpy(w).double()[:, None, :],
                                      padding=K // 2, groups=C).numpy()
    assert full.shape[-1] == L + 1
    y, ya = oracle_mod.fwd(x, w, K // 2)
    assert np.max(np.abs(y - full[..., :L]) / ya) < 1e-13


# ---------------------------------------------------------------- gradients: finite differences, adjoint identity
@pytest.mark.parametrize("B,C,L,K", [(2, 2, 9, 4), (1, 3, 6, 7), (2, 1, 12, 5)])
def test_finite_differences(oracle_mod, B, C, L, K):
    """phi = <dy, fwd(x,w)> is linear in x and in w, so central differences are exact up to rounding."""
    x = rnd((B, C, L), 11); w = rnd((C, K), 12); dy = rnd((B, C, L), 13)
    h = np.float32(0.5)     # exactly representable step: x +- h is exact in fp32 for |x| < 2^22

    def phi(xx, ww, p):
        y, _ = oracle_mod.fwd(xx, ww, p)
        return float((dy.astype(np.float64) * y).sum())

    for p in sorted({0, K // 2, K - 1}):
        dx, _ = oracle_mod.bwd_input(dy, w, p)
        dw, _ = oracle_mod.bwd_weight(x, dy, K, p)
        for idx in np.ndindex(B, C, L):
            xp = x.copy(); xm = x.copy()
            xp[idx] = np.float32(np.round(x[idx] * 4) / 4) + h
            xm[idx] = np.float32(np.round(x[idx] * 4) / 4) - h
            fd = (phi(xp, w, p) - phi(xm, w, p)) / (2.0 * float(h))
            assert abs(fd - dx[idx]) <= 1e-9 * max(1.0, abs(dx[idx])), (p, idx)
        for idx in np.ndindex(C, K):
            wp = w.copy(); wm = w.copy()
            wp[idx] = np.float32(np.round(w[idx] * 4) / 4) + h
            wm[idx] = np.float32(np.round(w[idx] * 4) / 4) - h
            fd = (phi(x, wp, p) - phi(x, wm, p)) / (2.0 * float(h))
            assert abs(fd - dw[idx]) <= 1e-9 * max(1.0, abs(dw[idx])), (p, idx)


@pytest.mark.parametrize("B,C,L,K", [(3, 4, 57, 16), (2, 2, 33, 48), (1, 5, 20, 33), (2, 3, 40, 1)])
def test_adjoint_identity(oracle_mod, B, C, L, K):
    x = rnd((B, C, L), 14); w = rnd((C, K), 15); dy = rnd((B, C, L), 16)
    for p in sorted({0, K // 2, (K - 1) // 2, K - 1}):
        y, ya = oracle_mod.fwd(x, w, p)
        dx, _ = oracle_mod.bwd_input(dy, w, p)
        dw, _ = oracle_mod.bwd_weight(x, dy, K, p)
        a = float((dy.astype(np.float64) * y).sum())
        b = float((dx * x.astype(np.float64)).sum())
        c = float((dw * w.astype(np.float64)).sum())
        scale = float((np.abs(dy.astype(np.float64)) * ya).sum())
        assert abs(a - b) <= 1e-13 * scale
        assert abs(a - c) <= 1e-13 * scale


def test_dx_is_forward_of_reversed_filter(oracle_mod):
    """dx = fwd(dy, reverse(w), pad_left = K-1-p): the same map written with the flipped filter of eq. (dx_def)."""
    B, C, L, K = 2, 3, 29, 10
    dy = rnd((B, C, L), 17); w = rnd((C, K), 18)
    wr = np.ascontiguousarray(w[:, ::-1])
    for p in all_pads(K):
        dx, dxa = oracle_mod.bwd_input(dy, w, p)
        y2, y2a = oracle_mod.fwd(dy, wr, K - 1 - p)
        np.testing.assert_allclose(dx, y2, rtol=0, atol=1e-13)
        np.testing.assert_allclose(dxa, y2a, rtol=0, atol=1e-13)


def printed_dx_def(dy, w, p):
    """Eq. (dx_def) exactly as printed: sum_j dy~[t+j-p] k[K-1-j]."""
    B, C, L = dy.shape
    K = w.shape[1]
    out = np.zeros((B, C, L))
    for t in range(L):
        for j in range(K):
            u = t + j - p
            if 0 <= u < L:
                out[:, :, t] += dy[:, :, u].astype(np.float64) * w[None, :, K - 1 - j].astype(np.float64)
    return out


def test_printed_dx_def_is_the_adjoint_for_odd_K_only(oracle_mod):
    B, C, L = 2, 2, 17
    dy = rnd((B, C, L), 19)
    for K in (3, 5, 9):
        w = rnd((C, K), 20)
        dx, _ = oracle_mod.bwd_input(dy, w, K // 2)
        np.testing.assert_allclose(dx, printed_dx_def(dy, w, K // 2), rtol=0, atol=1e-13)
    for K in (2, 4, 8):          # even K: printed offset is off by one from the gradient
        w = rnd((C, K), 21)
        dx, _ = oracle_mod.bwd_input(dy, w, K // 2)
        assert np.max(np.abs(dx - printed_dx_def(dy, w, K // 2))) > 1e-3


# ---------------------------------------------------------------- gradients: closed forms
def test_dx_identity_filter_is_shift(oracle_mod):
    B, C, L, K = 2, 2, 9, 5
    dy = rnd((B, C, L), 22)
    for p in all_pads(K):
        for j0 in range(K):
            w = np.zeros((C, K), np.float32); w[:, j0] = 1.0
            dx, _ = oracle_mod.bwd_input(dy, w, p)
            exp = np.zeros((B, C, L))
            for s in range(L):
                t = s - j0 + p
                if 0 <= t < L:
                    exp[:, :, s] = dy[:, :, t]
            assert np.array_equal(dx, exp)


def test_dw_delta_dy_reads_input_window(oracle_mod):
    B, C, L, K = 3, 2, 8, 6
    x = rnd((B, C, L), 23)
    for p in all_pads(K):
        for b0 in range(B):
            for t0 in (0, 3, L - 1):
                dy = np.zeros((B, C, L), np.float32); dy[b0, :, t0] = 1.0
                dw, _ = oracle_mod.bwd_weight(x, dy, K, p)
                for j in range(K):
                    u = t0 + j - p
                    exp = x[b0, :, u].astype(np.float64) if 0 <= u < L else np.zeros(C)
                    assert np.array_equal(dw[:, j], exp)


# ---------------------------------------------------------------- degenerate shapes, abs sums, channels, errors
def test_K_longer_than_L_and_K1(oracle_mod):
    B, C, L, K = 2, 2, 4, 11
    x = rnd((B, C, L), 24); w = rnd((C, K), 25); dy = rnd((B, C, L), 26)
    for p in all_pads(K):
        dw, dwa = oracle_mod.bwd_weight(x, dy, K, p)
        for j in range(K):
            if abs(j - p) >= L:            # tap never meets the input
                assert np.all(dw[:, j] == 0) and np.all(dwa[:, j] == 0)
    y, _ = oracle_mod.fwd(x, w[:, :1].copy(), 0)
    assert np.array_equal(y, x.astype(np.float64) * w[None, :, :1].astype(np.float64))


def test_abs_sums_are_values_of_absolute_inputs(oracle_mod):
    B, C, L, K, p = 2, 3, 21, 6, 4
    x = rnd((B, C, L), 27); w = rnd((C, K), 28); dy = rnd((B, C, L), 29)
    _, ya = oracle_mod.fwd(x, w, p)
    yv, _ = oracle_mod.fwd(np.abs(x), np.abs(w), p)
    np.testing.assert_allclose(ya, yv, rtol=1e-15)
    _, da = oracle_mod.bwd_input(dy, w, p)
    dv, _ = oracle_mod.bwd_input(np.abs(dy), np.abs(w), p)
    np.testing.assert_allclose(da, dv, rtol=1e-15)
    _, wa = oracle_mod.bwd_weight(x, dy, K, p)
    wv, _ = oracle_mod.bwd_weight(np.abs(x), np.abs(dy), K, p)
    np.testing.assert_allclose(wa, wv, rtol=1e-15)


def test_channels_do_not_interact(oracle_mod):
    """Depthwise: channel c of every output depends on channel c of the inputs only (Sec. IV-A)."""
    B, C, L, K, p = 2, 4, 15, 5, 2
    x = rnd((B, C, L), 30); w = rnd((C, K), 31); dy = rnd((B, C, L), 32)
    y, _ = oracle_mod.fwd(x, w, p)
    dw, _ = oracle_mod.bwd_weight(x, dy, K, p)
    x2 = x.copy(); x2[:, 1, :] += 1.0
    w2 = w.copy(); w2[1, :] *= 2.0
    y2, _ = oracle_mod.fwd(x2, w2, p)
    dw2, _ = oracle_mod.bwd_weight(x2, dy, K, p)
    keep = [0, 2, 3]
    assert np.array_equal(y[:, keep], y2[:, keep]) and not np.array_equal(y[:, 1], y2[:, 1])
    assert np.array_equal(dw[keep], dw2[keep]) and not np.array_equal(dw[1], dw2[1])


def test_oracle_rejects_bad_arguments(oracle_mod):
    x = rnd((1, 1, 4), 33); w = rnd((1, 3), 34)
    with pytest.raises(ValueError):
        oracle_mod.fwd(x, w, 3)
    with pytest.raises(ValueError):
        oracle_mod.bwd_input(x, w, -1)
    with pytest.raises(TypeError):
        oracle_mod.fwd(x.astype(np.float64), w, 1)
