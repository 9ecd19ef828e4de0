"""Pins for the combine oracle (CPU only): a hand-worked example with exactly representable values, torch float64
gather / sum, and the properties of a weighted sum."""
import numpy as np
import torch

import oracle
import workloads


def bits(a):
    return workloads.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_combine_hand_example():
    # four result rows of two values; three tokens with two slots each (Section 2.1, combine)
    y = bits([[1.0, -2.0], [0.5, 4.0], [8.0, 0.25], [-1.5, 3.0]])
    row_of = np.array([[2, 0], [1, 1], [3, -1]], dtype=np.int32)        # token 1 uses row 1 twice, token 2 lost its second expert
    gate = np.array([[0.5, 2.0], [0.25, 0.75], [4.0, 100.0]], dtype=np.float32)
    out = oracle.combine_topk_sum(y, row_of, gate)
    assert out.tolist() == [[0.5 * 8.0 + 2.0 * 1.0, 0.5 * 0.25 + 2.0 * -2.0], [0.5, 4.0], [-6.0, 12.0]]
    assert oracle.combine_topk_sum(y, row_of).tolist() == [[9.0, -1.75], [1.0, 8.0], [-1.5, 3.0]]      # no gate = unit weights
    # a row index past the end is treated like a dropped assignment
    assert oracle.combine_topk_sum(y, np.array([[4, 0]], dtype=np.int32)).tolist() == [[1.0, -2.0]]


def test_combine_matches_torch_gather_and_properties():
    rng = np.random.default_rng(3)
    R, d, T, topk = 60, 24, 17, 3
    y = workloads.activations(R, d, seed=9)
    row_of = rng.permutation(R)[:T * topk].reshape(T, topk).astype(np.int32)
    row_of[4, 1] = -1
    gate = rng.random((T, topk), dtype=np.float32)
    out = oracle.combine_topk_sum(y, row_of, gate)
    yt = torch.from_numpy(y.view(np.int16).copy()).view(torch.bfloat16).double()
    idx = torch.from_numpy(row_of.astype(np.int64)).clamp(min=0)
    w = torch.from_numpy(gate).double() * torch.from_numpy(row_of >= 0).double()
    ref = (yt[idx] * w[:, :, None]).sum(dim=1).numpy()
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-15) and np.abs(out).max() > 0.1
    # linear in the weights; the order of a token's slots does not matter; tokens do not influence each other
    assert np.allclose(oracle.combine_topk_sum(y, row_of, 2.0 * gate), 2.0 * out, rtol=1e-13)
    assert np.allclose(oracle.combine_topk_sum(y, row_of[:, ::-1], gate[:, ::-1]), out, rtol=1e-12, atol=1e-15)
    assert np.array_equal(oracle.combine_topk_sum(y, row_of[5:6], gate[5:6])[0], out[5])
    # a weight on the wrong slot changes the result
    assert not np.allclose(oracle.combine_topk_sum(y, row_of, gate[:, ::-1]), out)
