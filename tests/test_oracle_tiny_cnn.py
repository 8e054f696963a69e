"""Pins for the tiny-CNN oracle (glue layers in numpy float64 + the C convolutions + LARS)."""
import numpy as np

import oracle
from oracle import tiny_cnn
from paper_1709_05011_amd import synth


def _setup(batch=4):
    x = synth.normal((batch, 3, 32, 32), 1)
    labels = synth.uniform_int(batch, 2, 10)
    params = {
        "w1": synth.normal((16, 3, 3, 3), 3, std=float(np.sqrt(2 / 27))),
        "w2": synth.normal((32, 16, 3, 3), 4, std=float(np.sqrt(2 / 144))),
        "wf": synth.normal((10, 32), 5, std=float(np.sqrt(2 / 32))),
        "bf": np.zeros(10, dtype=np.float32),
    }
    return x, labels, params


def test_glue_layers_small_cases():
    x = np.array([[[[1., 5., 2., 2.], [3., 5., 2., 1.]]]])      # ties: first maximum wins
    y, idx = tiny_cnn.maxpool2(x)
    assert y.tolist() == [[[[5., 2.]]]] and idx.tolist() == [[[[1, 0]]]]
    dx = tiny_cnn.maxpool2_bwd(idx, np.array([[[[7., 9.]]]]), 2, 4)
    assert dx.tolist() == [[[[0., 7., 9., 0.], [0., 0., 0., 0.]]]]
    assert tiny_cnn.relu_bwd(np.array([-1., 0., 2.]), np.ones(3)).tolist() == [0., 0., 1.]
    loss, d = tiny_cnn.softmax_xent(np.zeros((2, 4)), np.array([1, 3]))
    assert abs(loss - np.log(4.0)) < 1e-15
    np.testing.assert_allclose(d, (np.full((2, 4), 0.25) - np.eye(4)[[1, 3]]) / 2)
    g = tiny_cnn.global_avgpool_bwd(np.array([[8.]]), 2, 2)
    assert g.tolist() == [[[[2., 2.], [2., 2.]]]]


def test_network_gradients_by_finite_differences():
    x, labels, params = _setup()
    t = tiny_cnn.forward_backward(x, labels, params)
    assert abs(t["loss"] - tiny_cnn.loss_only(x, labels, params)) < 1e-5
    h = 1e-4
    for name, seed in [("w1", 10), ("w2", 11), ("wf", 12), ("bf", 13)]:
        shape = params[name].shape
        for idx in map(tuple, synth.sample_coords(8, shape + (1,) * (4 - len(shape)), seed)[:, :len(shape)]):
            p64 = {k: v.astype(np.float64) for k, v in params.items()}
            p64[name][idx] += h
            up = tiny_cnn.loss_only(x, labels, p64)
            p64[name][idx] -= 2 * h
            dn = tiny_cnn.loss_only(x, labels, p64)
            fd = (up - dn) / (2 * h)
            got = float(t["d_" + name][idx])
            assert abs(fd - got) <= 2e-4 * max(abs(fd), 1e-2), (name, idx, fd, got)


def test_train_step_applies_lars_to_the_four_tensors():
    x, labels, params = _setup()
    vel = {k: np.zeros_like(v) for k, v in params.items()}
    before = {k: v.copy() for k, v in params.items()}
    t = tiny_cnn.train_step(x, labels, params, vel, 0.001, 0.9, 5e-4, 1.0)
    assert t["trust"].shape == (4,)
    assert t["trust"][3] == 1.0                         # zero-initialised bias: ||w|| = 0 fallback
    for i, k in enumerate(["w1", "w2", "wf"]):
        nw, ng = t["norms"][i]
        lam = 0.001 * nw / (ng + 5e-4 * nw)
        assert abs(t["trust"][i] - lam) < 1e-12
        v_ref = lam * (t["d_" + k] + 5e-4 * before[k].astype(np.float64))
        np.testing.assert_allclose(vel[k], v_ref, rtol=1e-6, atol=1e-12)
        np.testing.assert_allclose(params[k], before[k] - v_ref, rtol=1e-6, atol=1e-12)


# ---- the glue definitions one by one (textbook values) ----

def test_relu_and_its_gradient_hand_values():
    x = np.array([-2.0, -0.0, 0.0, 0.5, 3.0])
    np.testing.assert_array_equal(tiny_cnn.relu(x), [0.0, 0.0, 0.0, 0.5, 3.0])
    np.testing.assert_array_equal(tiny_cnn.relu_bwd(x, np.array([1.0, 2.0, 3.0, 4.0, 5.0])), [0.0, 0.0, 0.0, 4.0, 5.0])


def test_maxpool_hand_example_first_maximum_wins():
    x = np.array([[[[1.0, 5.0, 2.0, 2.0],
                    [5.0, 0.0, 2.0, 2.0],
                    [-1.0, -3.0, 0.0, 7.0],
                    [-2.0, -0.5, 8.0, 7.5]]]])
    y, idx = tiny_cnn.maxpool2(x)
    np.testing.assert_array_equal(y[0, 0], [[5.0, 2.0], [-0.5, 8.0]])
    np.testing.assert_array_equal(idx[0, 0], [[1, 0], [3, 2]])          # ties: position 1 before 2, 0 before the rest
    dx = tiny_cnn.maxpool2_bwd(idx, np.array([[[[10.0, 20.0], [30.0, 40.0]]]]), 4, 4)
    want = np.zeros((4, 4))
    want[0, 1], want[0, 2], want[3, 1], want[3, 2] = 10.0, 20.0, 30.0, 40.0
    np.testing.assert_array_equal(dx[0, 0], want)


def test_global_average_pool_is_the_mean_and_spreads_its_gradient_evenly():
    x = np.arange(2 * 3 * 2 * 5, dtype=np.float64).reshape(2, 3, 2, 5)
    y = tiny_cnn.global_avgpool(x)
    assert y[1, 2] == np.mean(np.arange(50, 60))
    dx = tiny_cnn.global_avgpool_bwd(np.ones((2, 3)) * 10.0, 2, 5)
    assert dx.shape == (2, 3, 2, 5) and np.all(dx == 1.0)


def test_softmax_cross_entropy_closed_forms():
    n, k = 4, 10
    loss, d = tiny_cnn.softmax_xent(np.full((n, k), 3.7), np.array([0, 3, 9, 3]))   # equal logits: p = 1/k
    assert abs(loss - np.log(k)) < 1e-12
    onehot = np.eye(k)[[0, 3, 9, 3]]
    np.testing.assert_allclose(d, (np.full((n, k), 1.0 / k) - onehot) / n, atol=1e-15)
    # two classes: loss = log(1 + exp(-(z_label - z_other)))
    z = np.array([[2.0, -1.0], [0.5, 0.25]])
    loss, d = tiny_cnn.softmax_xent(z, np.array([0, 1]))
    want = (np.log1p(np.exp(-3.0)) + np.log1p(np.exp(0.25))) / 2
    assert abs(loss - want) < 1e-12
    assert np.allclose(d.sum(axis=1), 0.0, atol=1e-15)
    # shifting a row's logits changes nothing
    loss2, d2 = tiny_cnn.softmax_xent(z + np.array([[100.0], [-50.0]]), np.array([0, 1]))
    assert abs(loss2 - loss) < 1e-12 and np.allclose(d2, d, atol=1e-14)
