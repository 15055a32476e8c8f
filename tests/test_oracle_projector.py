"""Pins for the oracle's feature projector (Algorithm 1: f = feature_projector(h); Sec. 3.1).

The paper fixes the network as two MLP layers; pooling, activation and normalisation are this
build's reading.  Each test checks the oracle against something fixed outside it: a hand-worked
case, a closed form, an invariant, or a library routine.
"""
import numpy as np
import pytest
import torch


def test_hand_worked_projection(oracle_mod):
    # two tokens [1,3] and [3,5]: mean x = [2,4]
    h = np.array([[[1, 3], [3, 5]]], np.float32)
    # asymmetric weights, so that a transposed operand gives other numbers
    W1 = np.array([[1, 2], [0, -1]], np.float32)
    b1 = np.array([0.5, 1.0], np.float32)
    # first layer: [1*2+2*4+0.5, 0*2-1*4+1] = [10.5, -3] -> ReLU -> [10.5, 0]
    W2 = np.array([[2, 1], [-1, 3]], np.float32)
    b2 = np.array([1.0, -1.0], np.float32)
    # second layer: [2*10.5+1*0+1, -10.5+0-1] = [22, -11.5]
    f = oracle_mod.project(h, W1, b1, W2, b2, normalize=False)
    assert f.tolist() == [[22.0, -11.5]]
    fn = oracle_mod.project(h, W1, b1, W2, b2, normalize=True)
    norm = (22.0 ** 2 + 11.5 ** 2) ** 0.5
    np.testing.assert_allclose(fn, [[22.0 / norm, -11.5 / norm]], rtol=1e-15)
    # only the first token counts when the sentence has one token: x = [1,3]
    # first layer [1+6+0.5, -3+1] = [7.5, -2] -> [7.5, 0]; second [16, -8.5]
    f1 = oracle_mod.project(h, W1, b1, W2, b2, seq_len=[1], normalize=False)
    assert f1.tolist() == [[16.0, -8.5]]
    # missing biases are zeros: [1*2+2*4, -4] -> [10, 0] -> [20, -10]
    f0 = oracle_mod.project(h, W1, None, W2, None, normalize=False)
    assert f0.tolist() == [[20.0, -10.0]]


def test_against_library_layers(oracle_mod):
    rng = np.random.default_rng(7)
    B, S, dm, hid, E = 5, 9, 24, 13, 6
    h = rng.standard_normal((B, S, dm)).astype(np.float32)
    W1 = rng.standard_normal((hid, dm)).astype(np.float32)
    b1 = rng.standard_normal(hid).astype(np.float32)
    W2 = rng.standard_normal((E, hid)).astype(np.float32)
    b2 = rng.standard_normal(E).astype(np.float32)
    sl = np.array([9, 1, 4, 7, 2], np.int32)
    t = lambda a: torch.from_numpy(a).double()
    mask = (torch.arange(S)[None, :] < torch.from_numpy(sl)[:, None]).double()
    x = (t(h) * mask[:, :, None]).sum(1) / torch.from_numpy(sl)[:, None].double()
    u = torch.relu(torch.nn.functional.linear(x, t(W1), t(b1)))
    f = torch.nn.functional.linear(u, t(W2), t(b2))
    got = oracle_mod.project(h, W1, b1, W2, b2, seq_len=sl, normalize=False)
    np.testing.assert_allclose(got, f.numpy(), rtol=1e-12, atol=1e-12)
    gotn = oracle_mod.project(h, W1, b1, W2, b2, seq_len=sl, normalize=True)
    np.testing.assert_allclose(gotn, torch.nn.functional.normalize(f, dim=1).numpy(),
                               rtol=1e-12, atol=1e-12)
    # without seq_len every token counts
    got_all = oracle_mod.project(h, W1, b1, W2, b2, normalize=False)
    f_all = torch.nn.functional.linear(
        torch.relu(torch.nn.functional.linear(t(h).mean(1), t(W1), t(b1))), t(W2), t(b2))
    np.testing.assert_allclose(got_all, f_all.numpy(), rtol=1e-12, atol=1e-12)


def test_signed_identity_layers_return_the_token_mean(oracle_mod):
    # W1 = [I; -I], W2 = [I, -I]: f = relu(x) - relu(-x) = x, so the output is the pooling itself
    rng = np.random.default_rng(3)
    B, S, dm = 3, 7, 8
    h = rng.standard_normal((B, S, dm)).astype(np.float32)
    eye = np.eye(dm, dtype=np.float32)
    W1 = np.concatenate([eye, -eye], 0)
    W2 = np.concatenate([eye, -eye], 1)
    f = oracle_mod.project(h, W1, None, W2, None, normalize=False)
    np.testing.assert_allclose(f, h.astype(np.float64).mean(1), rtol=1e-13, atol=1e-13)
    # and a layer of -I alone is cut to nothing by the activation wherever x > 0
    f = oracle_mod.project(np.abs(h), -eye, None, eye, None, normalize=False)
    assert np.all(f == 0.0)


def test_invariants(oracle_mod):
    rng = np.random.default_rng(11)
    B, S, dm, hid, E = 4, 10, 16, 12, 8
    h = rng.standard_normal((B, S, dm)).astype(np.float32)
    W1 = rng.standard_normal((hid, dm)).astype(np.float32)
    W2 = rng.standard_normal((E, hid)).astype(np.float32)
    b1 = rng.standard_normal(hid).astype(np.float32)
    b2 = rng.standard_normal(E).astype(np.float32)
    sl = np.array([10, 6, 3, 8], np.int32)
    base = oracle_mod.project(h, W1, b1, W2, b2, seq_len=sl)
    # unit norm
    np.testing.assert_allclose(np.linalg.norm(base, axis=1), 1.0, rtol=1e-14)
    # tokens past the sentence's length do not count
    h2 = h.copy()
    for b in range(B):
        h2[b, sl[b]:] = 1e6
    assert np.array_equal(oracle_mod.project(h2, W1, b1, W2, b2, seq_len=sl), base)
    # the order of the valid tokens does not matter (up to summation order)
    h3 = h.copy()
    for b in range(B):
        h3[b, :sl[b]] = h[b, rng.permutation(sl[b])]
    np.testing.assert_allclose(oracle_mod.project(h3, W1, b1, W2, b2, seq_len=sl), base,
                               rtol=1e-12, atol=1e-13)
    # without biases the network is positively homogeneous: f(c h) = c f(h), c > 0 a power of two
    f1 = oracle_mod.project(h, W1, None, W2, None, normalize=False)
    f4 = oracle_mod.project(4 * h, W1, None, W2, None, normalize=False)
    assert np.array_equal(f4, 4 * f1)
    # queries are independent of each other
    solo = oracle_mod.project(h[2:3], W1, b1, W2, b2, seq_len=sl[2:3])
    assert np.array_equal(solo[0], base[2])


def test_degenerate_cases(oracle_mod):
    h = np.ones((2, 3, 4), np.float32)
    W1 = np.zeros((5, 4), np.float32)
    W2 = np.ones((6, 5), np.float32)
    # a zero feature vector stays zero under normalisation
    f = oracle_mod.project(h, W1, None, W2, None, normalize=True)
    assert f.shape == (2, 6) and np.all(f == 0.0)
    # empty batch
    assert oracle_mod.project(np.zeros((0, 3, 4), np.float32), W1, None, W2, None).shape == (0, 6)
    with pytest.raises(RuntimeError):
        oracle_mod.project(h, W1, None, W2, None, seq_len=[0, 3])
    with pytest.raises(RuntimeError):
        oracle_mod.project(h, W1, None, W2, None, seq_len=[1, 4])
    with pytest.raises(ValueError):
        oracle_mod.project(h, np.zeros((5, 3), np.float32), None, W2, None)
