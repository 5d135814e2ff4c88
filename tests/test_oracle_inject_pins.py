"""Pins for the oracle of the gated target-feature injection (Sec.3.3): torch's linear layer
and autograd as an independent library definition, a hand-evaluated case, gate special cases.
CPU only."""
import numpy as np
import pytest

from oracle import inject_oracle as I


def _case(seed, T=7, d=5, dt=4, F=3):
    rng = np.random.default_rng(seed)
    E = rng.standard_normal((T, d))
    feats = [rng.standard_normal((T, dt)) for _ in range(F)]
    P = rng.standard_normal((d, F * dt))
    xi = (rng.random(T) < 0.7).astype(np.float64)
    return E, feats, P, xi


def test_hand_example():
    # one token, d = 2, two features of width 1: x = (2, 3); P = [[1, 10], [0.5, -1]]
    #   t = (2*1 + 3*10, 2*0.5 - 3) = (32, -2);  e = (1, 1):  gate 1 -> (33, -1), gate 0 -> (1, 1)
    E = np.array([[1.0, 1.0]])
    feats = [np.array([[2.0]]), np.array([[3.0]])]
    P = np.array([[1.0, 10.0], [0.5, -1.0]])
    np.testing.assert_allclose(I.inject_forward(E, feats, P, np.array([1.0])), [[33.0, -1.0]])
    np.testing.assert_allclose(I.inject_forward(E, feats, P, np.array([0.0])), [[1.0, 1.0]])
    # upstream gradient (1, 2), gate 1: dP = outer((1, 2), (2, 3))
    dT, dP = I.inject_backward(np.array([[1.0, 2.0]]), feats, np.array([1.0]))
    np.testing.assert_allclose(dT, [[1.0, 2.0]])
    np.testing.assert_allclose(dP, [[2.0, 3.0], [4.0, 6.0]])


def test_vs_torch_linear_and_autograd():
    torch = pytest.importorskip("torch")
    E, feats, P, xi = _case(1)
    Pt = torch.tensor(P, requires_grad=True)
    Et = torch.tensor(E, requires_grad=True)
    X = torch.cat([torch.tensor(f) for f in feats], dim=1)
    out = Et + torch.tensor(xi)[:, None] * torch.nn.functional.linear(X, Pt)
    np.testing.assert_allclose(I.inject_forward(E, feats, P, xi), out.detach().numpy(), atol=1e-13)
    G = np.random.default_rng(2).standard_normal(E.shape)
    out.backward(torch.tensor(G))
    dT, dP = I.inject_backward(G, feats, xi)
    np.testing.assert_allclose(dP, Pt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(Et.grad.numpy(), G)                      # dE is the identity
    np.testing.assert_allclose(dT, xi[:, None] * G)


def test_gate_special_cases_and_concat_order():
    E, feats, P, xi = _case(3)
    T = E.shape[0]
    np.testing.assert_array_equal(I.inject_forward(E, feats, P, np.zeros(T)), E)     # rho = 1: never injected
    full = I.inject_forward(E, feats, P, np.ones(T))
    gated = I.inject_forward(E, feats, P, xi)
    np.testing.assert_allclose(gated, np.where(xi[:, None] > 0, full, E))
    # the projection's column blocks follow the order of the features
    dt = feats[0].shape[1]
    parts = sum(f @ P[:, i * dt:(i + 1) * dt].T for i, f in enumerate(feats))
    np.testing.assert_allclose(full - E, parts, atol=1e-13)
    swapped = I.inject_forward(E, feats[::-1], P, np.ones(T))
    assert np.abs(swapped - full).max() > 1e-3
    _, dP = I.inject_backward(np.ones_like(E), feats, np.zeros(T))
    assert not dP.any()
