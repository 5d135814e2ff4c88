"""Pins for the fp64 oracle of the weighted (beta CE + KD) loss (Eq.12 under the forward-KL
reading): a hand-evaluated token, scipy's entropy routine and torch autograd as independent
library definitions, closed forms, the teacher == draft reduction to the CE-only oracle,
finite differences.  CPU only.
"""
import os

import numpy as np
import pytest
from scipy.special import log_softmax, softmax
from scipy.stats import entropy

from oracle import cat_kd_oracle as KD
from oracle import cat_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(seed, B=3, K=4, d=6, dt=9, V=17, scale=1.5):
    rng = np.random.default_rng(seed)
    T = B * K
    H = rng.standard_normal((T, d))
    W = rng.standard_normal((V, d)) * scale / np.sqrt(d)
    Ht = rng.standard_normal((T, dt))
    Wt = rng.standard_normal((V, dt)) * scale / np.sqrt(dt)
    y = rng.integers(0, V, size=T)
    return H, W, Ht, Wt, y


def _golden():
    out = {}
    with open(os.path.join(GOLDEN, "eq12_kd_hand_example.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                out[key] = np.array([float(v) for v in vals])
    return out


def test_hand_example_token():
    gold = _golden()
    H = np.array([[1.0]]); W = np.array([[0.0], [0.0]])
    Ht = np.array([[1.0]]); Wt = np.array([[np.log(3.0)], [0.0]])
    y = np.array([0])
    beta = float(gold["beta"][0])
    f = KD.cat_kd_loss_and_grads(H, W, Ht, Wt, y, B=1, K=1, beta=beta)
    assert abs(f["kd"][0] - gold["kd"][0]) < 1e-9
    assert abs(-f["logq"][0] - gold["ce"][0]) < 1e-9
    assert abs(f["loss"] - gold["loss"][0]) < 1e-9
    assert abs(f["conf"][0] - gold["conf"][0]) < 1e-12
    np.testing.assert_allclose(f["dW"][:, 0], gold["dZ"], atol=1e-12)     # h = 1: dW = dZ
    np.testing.assert_allclose(f["dH"], 0.0, atol=1e-15)                  # draft head is zero


def test_kd_matches_scipy_entropy_and_is_directional():
    H, W, Ht, Wt, y = tiny(3)
    st = KD.kd_stats(H, W, Ht, Wt, y)
    P = softmax(Ht @ Wt.T, axis=1)
    Q = softmax(H @ W.T, axis=1)
    for t in range(len(y)):
        assert abs(st["kd"][t] - entropy(P[t], Q[t])) < 1e-12          # KL(p || q)
        assert abs(st["kd"][t] - entropy(Q[t], P[t])) > 1e-3           # not the reverse
    assert np.all(st["kd"] > 0)
    np.testing.assert_allclose(st["logp_t"], log_softmax(Ht @ Wt.T, axis=1)[np.arange(len(y)), y], atol=1e-12)
    np.testing.assert_allclose(st["logq"], log_softmax(H @ W.T, axis=1)[np.arange(len(y)), y], atol=1e-12)


def test_teacher_equal_to_draft_reduces_to_self_teacher_ce():
    H, W, _, _, y = tiny(4)
    B, K, beta = 3, 4, 0.3
    f = KD.cat_kd_loss_and_grads(H, W, H, W, y, B, K, beta=beta)
    ref = O.cat_loss_and_grads(H, W, y, B, K, beta=beta)                 # self-teacher CE-only oracle
    np.testing.assert_allclose(f["kd"], 0.0, atol=1e-13)
    assert abs(f["loss"] - ref["loss"]) < 1e-13
    np.testing.assert_allclose(f["w"], ref["w"], rtol=1e-13)
    np.testing.assert_allclose(f["dH"], ref["dH"], atol=1e-14)
    np.testing.assert_allclose(f["dW"], ref["dW"], atol=1e-14)


def test_uniform_teacher_closed_form():
    H, W, Ht, Wt, y = tiny(5)
    V = W.shape[0]
    st = KD.kd_stats(H, W, Ht, np.zeros_like(Wt), y)
    logQ = log_softmax(H @ W.T, axis=1)
    np.testing.assert_allclose(st["kd"], -np.log(V) - logQ.mean(axis=1), atol=1e-12)
    np.testing.assert_allclose(st["logp_t"], -np.log(V), atol=1e-12)


def test_default_confidence_is_teacher_probability_eq9():
    H, W, Ht, Wt, y = tiny(6)
    B, K = 3, 4
    f = KD.cat_kd_forward(H, W, Ht, Wt, y, B, K)
    P = softmax(Ht @ Wt.T, axis=1)
    c = P[np.arange(B * K), y].reshape(B, K)
    for b in range(B):
        for k in range(K):
            assert abs(f["w"][b * K + k] - np.prod(c[b, :k])) < 1e-14   # Eq.10 over Eq.9
    ext = np.random.default_rng(0).random(B * K)
    f2 = KD.cat_kd_forward(H, W, Ht, Wt, y, B, K, conf_in=ext)
    s, _ = O.cat_weights(ext, B, K)
    np.testing.assert_allclose(f2["w"], s)


@pytest.mark.parametrize("beta,reduction", [(0.1, O.RED_MEAN_VALID), (1.0, O.RED_SUM)])
def test_loss_and_grads_vs_torch_autograd(beta, reduction):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    H, W, Ht, Wt, y = tiny(7)
    B, K = 3, 4
    vl = np.array([4, 2, 3])
    y = y.copy(); y[1] = -100
    f = KD.cat_kd_loss_and_grads(H, W, Ht, Wt, y, B, K, valid_len=vl, beta=beta, reduction=reduction, gout=1.7)
    Hd = torch.tensor(H, requires_grad=True); Wd = torch.tensor(W, requires_grad=True)
    zt = torch.tensor(Ht @ Wt.T)
    logq = F.log_softmax(Hd @ Wd.T, dim=1)
    kd = F.kl_div(logq, F.softmax(zt, dim=1), reduction="none").sum(dim=1)
    valid = O.valid_mask(y, B, K, vl)
    ys = torch.tensor(np.where(y < 0, 0, y))
    ce = -logq[torch.arange(B * K), ys]
    w = torch.tensor(f["w"])                                           # constant weights
    tok = torch.where(torch.tensor(valid), w * (beta * ce + kd), torch.zeros_like(ce))
    loss = tok.sum() / (valid.sum() if reduction == O.RED_MEAN_VALID else 1.0)
    (1.7 * loss).backward()
    assert abs(float(loss.detach()) - f["loss"]) < 1e-12
    np.testing.assert_allclose(f["dH"], Hd.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(f["dW"], Wd.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(f["kd"], kd.detach().numpy(), atol=1e-12)


def test_finite_differences_of_the_whole_forward():
    # the weights depend on the teacher only, so the plain derivative of the forward with
    # respect to the draft's H and W is the analytic gradient: nothing needs freezing
    H, W, Ht, Wt, y = tiny(8, B=2, K=3, d=4, dt=5, V=9)
    B, K, beta = 2, 3, 0.4
    f = KD.cat_kd_loss_and_grads(H, W, Ht, Wt, y, B, K, beta=beta)
    eps = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(6):
        t, i = rng.integers(0, B * K), rng.integers(0, 4)
        Hp, Hm = H.copy(), H.copy(); Hp[t, i] += eps; Hm[t, i] -= eps
        fd = (KD.cat_kd_forward(Hp, W, Ht, Wt, y, B, K, beta=beta)["loss"]
              - KD.cat_kd_forward(Hm, W, Ht, Wt, y, B, K, beta=beta)["loss"]) / (2 * eps)
        assert abs(fd - f["dH"][t, i]) < 1e-7 * max(1.0, abs(fd))
        v = rng.integers(0, 9)
        Wp, Wm = W.copy(), W.copy(); Wp[v, i] += eps; Wm[v, i] -= eps
        fd = (KD.cat_kd_forward(H, Wp, Ht, Wt, y, B, K, beta=beta)["loss"]
              - KD.cat_kd_forward(H, Wm, Ht, Wt, y, B, K, beta=beta)["loss"]) / (2 * eps)
        assert abs(fd - f["dW"][v, i]) < 1e-7 * max(1.0, abs(fd))


def test_gradient_invariants_and_sampling():
    H, W, Ht, Wt, y = tiny(9)
    B, K = 3, 4
    f = KD.cat_kd_loss_and_grads(H, W, Ht, Wt, y, B, K, beta=0.2)
    np.testing.assert_allclose(f["dW"].sum(axis=0), 0.0, atol=1e-14)      # sum_v dZ[t,v] = 0 for every t
    rows, vrows = np.array([1, 7, 10]), np.array([0, 5, 16, int(y[2])])
    part = KD.cat_kd_backward(H, W, Ht, Wt, y, f["lse"], f["lse_t"], f["g"], 0.2, rows=rows, vrows=vrows)
    np.testing.assert_allclose(part["dH"], f["dH"][rows], atol=1e-15)
    np.testing.assert_allclose(part["dW"], f["dW"][vrows], atol=1e-15)
    sub = KD.kd_stats(H, W, Ht, Wt, y, rows=rows)
    np.testing.assert_allclose(sub["kd"], f["kd"][rows], atol=1e-15)


def test_all_ignored_gives_zero():
    H, W, Ht, Wt, y = tiny(10)
    f = KD.cat_kd_loss_and_grads(H, W, Ht, Wt, np.full_like(y, -100), 3, 4)
    assert f["loss"] == 0.0 and not f["dH"].any() and not f["dW"].any()
