"""Pins for the batch-normalisation oracle: a hand-worked channel, the statistics of its output, invariances,
and its gradient against central finite differences of the forward definition.  No HIP path here."""
import numpy as np

from oracle import batchnorm as bn
from paper_1709_05011_amd import synth


def test_hand_worked_channel():
    # one channel, values 1, 2, 3, 6: mean 3, biased variance (4 + 1 + 0 + 9)/4 = 3.5
    x = np.array([1.0, 2.0, 3.0, 6.0]).reshape(2, 1, 1, 2)
    y, mean, inv_std = bn.forward(x, [2.0], [0.5], eps=0.0)
    assert mean[0] == 3.0 and abs(inv_std[0] - 1 / np.sqrt(3.5)) < 1e-15
    np.testing.assert_allclose(y.reshape(-1), 2.0 * (np.array([1, 2, 3, 6]) - 3.0) / np.sqrt(3.5) + 0.5, atol=1e-14)
    # eps enters under the root
    _, _, inv2 = bn.forward(x, [2.0], [0.5], eps=0.5)
    assert abs(inv2[0] - 0.5) < 1e-15


def test_output_statistics_and_invariances():
    x = synth.normal((6, 5, 7, 3), 8100).astype(np.float64) * 3.0 + 1.5
    gamma = np.array([1.0, 2.0, 0.5, -1.0, 3.0])
    beta = np.array([0.0, 1.0, -2.0, 0.25, 4.0])
    y, mean, inv_std = bn.forward(x, gamma, beta, eps=0.0)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), beta, atol=1e-12)             # mean beta, std |gamma|
    np.testing.assert_allclose(y.std(axis=(0, 2, 3)), np.abs(gamma), atol=1e-12)
    # shifting or scaling the input of a channel changes nothing (eps = 0)
    y2, _, _ = bn.forward(x * 7.0 + 11.0, gamma, beta, eps=0.0)
    np.testing.assert_allclose(y2, y, atol=1e-11)
    # channels are independent: permuting them permutes the output
    perm = [3, 0, 4, 1, 2]
    y3, _, _ = bn.forward(x[:, perm], gamma[perm], beta[perm], eps=0.0)
    np.testing.assert_allclose(y3, y[:, perm], atol=1e-13)


def test_gradient_against_finite_differences():
    x = synth.normal((3, 2, 4, 2), 8200).astype(np.float64)
    dy = synth.normal((3, 2, 4, 2), 8201).astype(np.float64)
    gamma, beta, eps = np.array([1.5, -0.75]), np.array([0.1, 0.2]), 1e-3
    loss = lambda xx, gg, bb: float(np.sum(bn.forward(xx, gg, bb, eps)[0] * dy))
    dx, dgamma, dbeta = bn.backward(x, dy, gamma, eps)
    h = 1e-6
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        num[idx] = (loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * h)
    np.testing.assert_allclose(dx, num, rtol=1e-6, atol=1e-8)
    for c in range(2):
        e = np.zeros(2)
        e[c] = h
        assert abs((loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h) - dgamma[c]) < 1e-7
        assert abs((loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h) - dbeta[c]) < 1e-7
    # the input gradient of a channel sums to zero and is orthogonal to the normalised input (eps aside)
    dx0, _, _ = bn.backward(x, dy, gamma, 0.0)
    assert np.allclose(dx0.sum(axis=(0, 2, 3)), 0.0, atol=1e-12)
    xhat = (x - x.mean(axis=(0, 2, 3), keepdims=True)) / x.std(axis=(0, 2, 3), keepdims=True)
    assert np.allclose((dx0 * xhat).sum(axis=(0, 2, 3)), 0.0, atol=1e-12)
