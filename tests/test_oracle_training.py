"""Pins for the oracle's loss, gradient sum and update (Alg. 1 last line, Alg. 2 first and
last lines): library log-softmax / cross-entropy, closed forms, finite differences."""
import numpy as np
import pytest
import torch


def test_loss_matches_library_cross_entropy(oracle):
    rng = np.random.default_rng(0)
    n, C = 500, 41
    H = (rng.standard_normal((n, C)) * 3).astype(np.float32)
    y = rng.integers(0, C, n).astype(np.int32)
    y[rng.random(n) < 0.4] = -1                       # unlabelled rows
    count = 777.0                                       # labelled nodes of the whole graph
    loss, J = oracle.softmax_xent(H, y, count)
    lab = y >= 0
    Ht = torch.from_numpy(H[lab]).double().requires_grad_(True)
    ref = torch.nn.functional.cross_entropy(Ht, torch.from_numpy(y[lab]).long(), reduction="sum") / count
    ref.backward()
    assert abs(loss - ref.item()) <= 1e-12 * abs(ref.item())
    assert np.array_equal(J[~lab], np.zeros_like(J[~lab]))
    assert np.allclose(J[lab], Ht.grad.numpy(), rtol=0, atol=2e-7 / count)
    assert np.array_equal(J[lab], Ht.grad.numpy().astype(np.float32))


def test_loss_closed_forms(oracle):
    C = 7
    H = np.zeros((4, C), np.float32)                   # uniform logits: loss = log C
    y = np.array([0, 3, 6, -1], np.int32)
    loss, J, S = oracle.softmax_xent(H, y, 3.0, want_S=True)
    assert abs(loss - np.log(C)) < 1e-15
    assert np.allclose(J[:3].astype(np.float64).sum(1), 0, atol=1e-7)     # gradient rows sum to zero
    assert np.allclose(J[0, 1:], 1 / C / 3) and np.isclose(J[0, 0], (1 / C - 1) / 3)
    assert np.allclose(S[0, 1:], 1 / C / 3) and np.isclose(S[0, 0], (1 / C + 1) / 3)
    assert not J[3].any() and not S[3].any()
    # a confidently right row costs nothing, a confidently wrong one its margin; shift invariance
    H = np.array([[50, 0, 0], [0, 50, 0]], np.float32)
    loss, J = oracle.softmax_xent(H, np.array([0, 0], np.int32), 2.0)
    assert abs(loss - 25.0) < 1e-9
    l2, J2 = oracle.softmax_xent(H + np.float32(1000), np.array([0, 0], np.int32), 2.0)
    assert abs(l2 - loss) < 1e-9 and np.array_equal(J, J2)


def test_loss_gradient_by_finite_differences(oracle):
    rng = np.random.default_rng(1)
    H = rng.standard_normal((6, 5)).astype(np.float32)
    y = np.array([1, 4, -1, 0, 2, 2], np.int32)
    _, J = oracle.softmax_xent(H, y, 5.0)
    eps = np.float32(2.0 ** -7)
    for i, c in ((0, 1), (1, 2), (3, 0), (5, 4), (2, 3)):
        Hp, Hm = H.copy(), H.copy()
        Hp[i, c] += eps; Hm[i, c] -= eps
        fd = (oracle.softmax_xent(Hp, y, 5.0)[0] - oracle.softmax_xent(Hm, y, 5.0)[0]) / (2 * float(eps))
        assert abs(fd - J[i, c]) < 1e-5


def test_gradient_sum_and_update(oracle):
    rng = np.random.default_rng(2)
    gs = [(rng.standard_normal((13, 7)) * 10.0 ** rng.integers(-3, 4)).astype(np.float32) for _ in range(4)]
    s = oracle.sum_gradients(gs)
    ref = gs[0].copy()
    for g in gs[1:]:
        ref = ref + g                                   # numpy float32, same order
    assert np.array_equal(s, ref)
    assert not np.array_equal(s, ((gs[3] + gs[2]) + gs[1]) + gs[0])     # the order is observable
    assert np.array_equal(oracle.sum_gradients(gs[:1]), gs[0])
    W = rng.standard_normal((13, 7)).astype(np.float32)
    W0 = W.copy()
    oracle.sgd_update(W, s, 0.05)
    assert np.array_equal(W, W0 - np.float32(0.05) * s)
    # partition sums of the loss equal the unpartitioned loss when `count` is the global count
    H = rng.standard_normal((40, 6)).astype(np.float32)
    y = rng.integers(-1, 6, 40).astype(np.int32)
    cnt = float((y >= 0).sum())
    whole, Jw = oracle.softmax_xent(H, y, cnt)
    a, Ja = oracle.softmax_xent(H[:17].copy(), y[:17].copy(), cnt)
    b, Jb = oracle.softmax_xent(H[17:].copy(), y[17:].copy(), cnt)
    assert abs(whole - (a + b)) < 1e-12 and np.array_equal(Jw, np.concatenate([Ja, Jb]))
