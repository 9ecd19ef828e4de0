"""Pins for the backward oracle (CPU only): torch's reverse-mode differentiation of the forward expression in float64
(a library routine that shares nothing with the hand-derived formulas), a central finite difference of the forward
oracle, and the structure of the gradients."""
import numpy as np
import torch

import oracle
import workloads


def _dec(b):
    return torch.from_numpy(np.ascontiguousarray(b).view(np.int16).copy()).view(torch.bfloat16).double()


def test_backward_matches_torch_autograd():
    E_loc, d, f, M, S = 2, 128, 256, 90, 3
    W = workloads.ffn_weights(E_loc, d, f, seed=31)
    x = workloads.activations(M, d, seed=32)
    dy = workloads.activations(M, d, seed=33)
    offsets = workloads.random_offsets(S * E_loc, M, seed=34)
    dx, dWg, dWu, dWd = oracle.expert_ffn_backward_sliced(x, dy, offsets, E_loc, W)
    xt = _dec(x).requires_grad_(True)
    wg, wu, wd = (_dec(w).requires_grad_(True) for w in (W.w_gate, W.w_up, W.w_down))
    expert = torch.from_numpy((np.searchsorted(offsets, np.arange(M), side="right") - 1) % E_loc)
    y = torch.zeros((M, d), dtype=torch.float64)
    for e in range(E_loc):
        sel = torch.nonzero(expert == e).flatten()
        ye = (torch.nn.functional.silu(xt[sel] @ wg[e].T) * (xt[sel] @ wu[e].T)) @ wd[e].T
        y = y.index_add(0, sel, ye)
    (y * _dec(dy)).sum().backward()                                     # loss whose gradient with respect to y is dy
    for got, ref, name in ((dx, xt.grad, "dx"), (dWg, wg.grad, "dWg"), (dWu, wu.grad, "dWu"), (dWd, wd.grad, "dWd")):
        ref = ref.numpy()
        assert np.abs(ref).max() > 1e-3, name
        assert np.allclose(got, ref, rtol=1e-10, atol=1e-12 * np.abs(ref).max()), name


def test_backward_matches_finite_differences_of_the_forward_oracle():
    E_loc, d, f, M = 1, 128, 128, 6
    W = workloads.ffn_weights(E_loc, d, f, seed=41)
    x = workloads.activations(M, d, seed=42)
    dy = workloads.activations(M, d, seed=43)
    offsets = np.array([0, M], dtype=np.int32)
    dx, _, _, _ = oracle.expert_ffn_backward_sliced(x, dy, offsets, E_loc, W)
    # d/dx[m][i] of sum(y * dy) by a central difference on the float64 forward expression (x perturbed in float64)
    wg, wu, wd = (oracle.decode_bf16(w[0]) for w in (W.w_gate, W.w_up, W.w_down))
    xf, dyf = oracle.decode_bf16(x), oracle.decode_bf16(dy)

    def loss(xx):
        g, u = xx @ wg.T, xx @ wu.T
        return float((((g / (1.0 + np.exp(-g))) * u) @ wd.T * dyf).sum())
    rng = np.random.default_rng(0)
    for _ in range(12):
        m, i = int(rng.integers(M)), int(rng.integers(d))
        eps = 1e-5
        xp, xm = xf.copy(), xf.copy()
        xp[m, i] += eps
        xm[m, i] -= eps
        fd = (loss(xp) - loss(xm)) / (2 * eps)
        assert abs(fd - dx[m, i]) <= 1e-6 * max(1.0, abs(dx[m, i])), (m, i, fd, dx[m, i])


def test_backward_structure():
    E_loc, d, f, M = 2, 128, 128, 40
    W = workloads.ffn_weights(E_loc, d, f, seed=51)
    x = workloads.activations(M, d, seed=52)
    dy = workloads.activations(M, d, seed=53)
    off = np.array([0, 10, 25, 30, 40], dtype=np.int32)                  # 2 slices x 2 experts
    dx, dWg, dWu, dWd = oracle.expert_ffn_backward_sliced(x, dy, off, E_loc, W)
    # a row's dx depends only on the row and its expert; weight gradients add up over the slices of an expert
    order = np.concatenate([np.arange(0, 10), np.arange(25, 30), np.arange(10, 25), np.arange(30, 40)])    # expert-major
    off1 = np.array([0, 15, 40], dtype=np.int32)
    dx1, dWg1, dWu1, dWd1 = oracle.expert_ffn_backward_sliced(x[order], dy[order], off1, E_loc, W)
    assert np.allclose(dx1, dx[order], rtol=1e-12, atol=1e-15)
    for a, b in ((dWg, dWg1), (dWu, dWu1), (dWd, dWd1)):
        assert np.allclose(a, b, rtol=1e-11, atol=1e-13)
    # zero upstream gradient on a row: no dx there and no contribution to the weights
    dy0 = dy.copy()
    dy0[3] = 0
    dx0, dWg0, _, _ = oracle.expert_ffn_backward_sliced(x, dy0, off, E_loc, W)
    assert not dx0[3].any() and not np.allclose(dWg0[0], dWg[0])
    # doubling dy doubles every gradient (bf16 exponent bump)
    dy2 = (dy + np.uint16(1 << 7)).astype(np.uint16)
    dx2, dWg2, dWu2, dWd2 = oracle.expert_ffn_backward_sliced(x, dy2, off, E_loc, W)
    assert np.array_equal(dx2, 2 * dx) and np.array_equal(dWd2, 2 * dWd) and np.array_equal(dWg2, 2 * dWg)
