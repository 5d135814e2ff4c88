"""Pins for the fp64 oracle: everything here checks `oracle/` against something
other than itself — hand-evaluated definitions, closed forms, invariants the
paper's equations imply, library routines (scipy log-softmax, torch autograd) on
the degenerate cases where the CAT loss reduces to a textbook cross-entropy,
brute force and finite differences on tiny problems.  CPU only.
"""
import os

import numpy as np
import pytest
from scipy.special import log_softmax, logsumexp

from oracle import cat_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_problem(seed, B=3, K=4, d=6, V=17, scale=1.5):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((B * K, d))
    W = rng.standard_normal((V, d)) * scale / np.sqrt(d)
    y = rng.integers(0, V, size=B * K)
    return H, W, y


# ---------------------------------------------------------------- Eq.10 / Eq.8
def _read_hand_example():
    blocks, cur = [], {}
    with open(os.path.join(GOLDEN, "eq10_hand_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            cur[key] = np.array([float(v) for v in vals])
            if key == "exp_len":
                blocks.append(cur)
                cur = {}
    return blocks


def test_hand_example_eq10():
    blocks = _read_hand_example()
    conf = np.concatenate([b["conf"] for b in blocks])
    s, exp_len = O.cat_weights(conf, B=len(blocks), K=4)
    np.testing.assert_allclose(s, np.concatenate([b["s"] for b in blocks]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(exp_len, [b["exp_len"][0] for b in blocks], rtol=0, atol=1e-15)


def test_weights_bruteforce_product():
    rng = np.random.default_rng(1)
    B, K = 5, 7
    conf = rng.random(B * K)
    s, exp_len = O.cat_weights(conf, B, K)
    c = conf.reshape(B, K)
    for b in range(B):
        for k in range(K):
            assert abs(s[b * K + k] - np.prod(c[b, :k])) < 1e-15       # Eq.10 literally
        # Eq.3 == Eq.6 == Eq.8:  sum_k prod_{j<=k} c_j == sum_k s_k c_k
        assert abs(exp_len[b] - sum(np.prod(c[b, :k + 1]) for k in range(K))) < 1e-14


def test_weights_range_and_monotone():
    rng = np.random.default_rng(2)
    B, K = 64, 16
    conf = rng.random(B * K)
    s, _ = O.cat_weights(conf, B, K)
    s = s.reshape(B, K)
    assert np.all(s[:, 0] == 1.0)
    assert np.all((s >= 0) & (s <= 1))
    assert np.all(np.diff(s, axis=1) <= 0)                 # non-increasing along the prefix
    np.testing.assert_allclose(s[:, 1:], s[:, :-1] * conf.reshape(B, K)[:, :-1], rtol=1e-15)


def test_last_conf_never_enters_a_weight():
    conf = np.array([0.3, 0.6, 0.9, 0.2])
    s1, _ = O.cat_weights(conf, 1, 4)
    conf[3] = 0.99
    s2, _ = O.cat_weights(conf, 1, 4)
    assert np.array_equal(s1, s2)


def test_decay_and_uniform_modes():
    s, _ = O.cat_weights(np.full(8, 0.5), 2, 4, mode=O.W_DECAY, gamma=0.8)
    np.testing.assert_allclose(s.reshape(2, 4), [[1, 0.8, 0.64, 0.512]] * 2, rtol=1e-15)
    s, _ = O.cat_weights(np.full(8, 0.5), 2, 4, mode=O.W_UNIFORM)
    assert np.all(s == 1.0)


def test_exp_len_respects_valid_len():
    conf = np.array([0.9, 0.5, 0.8, 0.25])
    _, e = O.cat_weights(conf, 1, 4, valid_len=[2])
    assert abs(e[0] - (0.9 + 0.45)) < 1e-15


# ------------------------------------------------------------ softmax statistics
def test_head_stats_vs_scipy():
    H, W, y = tiny_problem(3, B=4, K=4, d=8, V=33)
    st = O.head_stats(H, W, y)
    Z = np.einsum("ti,vi->tv", H, W)                  # independent contraction routine
    np.testing.assert_allclose(st["lse"], logsumexp(Z, axis=1), rtol=1e-14)
    np.testing.assert_allclose(st["logq"], log_softmax(Z, axis=1)[np.arange(16), y], rtol=1e-12, atol=1e-14)
    assert np.array_equal(st["argmax"], Z.argmax(axis=1))
    assert np.all(st["logq"] <= 0)
    q = np.exp(Z - st["lse"][:, None])
    np.testing.assert_allclose(q.sum(axis=1), 1.0, atol=1e-12)
    srt = np.sort(Z, axis=1)
    np.testing.assert_allclose(st["gap"], srt[:, -1] - srt[:, -2], atol=1e-13)


def test_head_stats_transposed_operand_would_fail():
    # z = H W^T, not H^T-anything: with d != V != T the shapes pin the orientation,
    # and a non-symmetric hand case pins the index order.
    H = np.array([[1.0, 2.0]])
    W = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    np.testing.assert_allclose(O.head_logits(H, W), [[1.0, 2.0, 3.0]])
    st = O.head_stats(H, W, [1])
    assert st["argmax"][0] == 2
    assert abs(st["logq"][0] - (2.0 - np.log(np.e + np.e ** 2 + np.e ** 3))) < 1e-14


def test_argmax_lowest_index_on_ties():
    H = np.ones((2, 4))
    W = np.zeros((6, 4))
    W[2] = W[4] = 0.5
    st = O.head_stats(H, W, [0, 0])
    assert list(st["argmax"]) == [2, 2]
    assert np.all(st["gap"] == 0)


def test_zero_weight_closed_form():
    B, K, d, V = 3, 4, 5, 11
    rng = np.random.default_rng(4)
    H = rng.standard_normal((B * K, d))
    W = np.zeros((V, d))
    y = rng.integers(0, V, B * K)
    conf = rng.random(B * K)
    r = O.cat_loss_and_grads(H, W, y, B, K, conf_in=conf, beta=0.1)
    np.testing.assert_allclose(r["logq"], -np.log(V), rtol=1e-15)
    np.testing.assert_allclose(r["loss"], 0.1 * np.log(V) * r["w"].mean(), rtol=1e-14)
    assert np.all(r["argmax"] == 0)
    np.testing.assert_allclose(r["dH"], 0, atol=1e-18)
    # dW[v] = sum_t g_t (1/V - 1[v=y_t]) H[t]
    g = 0.1 * r["w"] / (B * K)
    expect = np.zeros((V, d))
    for t in range(B * K):
        for v in range(V):
            expect[v] += g[t] * (1.0 / V - (v == y[t])) * H[t]
    np.testing.assert_allclose(r["dW"], expect, atol=1e-16)


def test_one_hot_dominant_logits_give_zero_loss():
    V, d = 7, 7
    W = np.eye(V) * 60.0
    H = np.eye(d)[[1, 3, 5, 6]]
    r = O.cat_forward(H, W, [1, 3, 5, 6], 1, 4)
    assert r["loss"] < 1e-20 + 1e-12
    assert list(r["accept_len"]) == [4]
    np.testing.assert_allclose(r["exp_len"], 4.0, atol=1e-12)   # every c = 1 (self-teacher)


# ------------------------------------------------ degenerate cases -> textbook CE
def _mean_nll(H, W, y):
    return float(-np.mean(log_softmax(H @ W.T, axis=1)[np.arange(len(y)), y]))


@pytest.mark.parametrize("case", ["conf_one", "k_one", "decay_gamma_one", "uniform"])
def test_degenerate_reduces_to_uniform_ce(case):
    H, W, y = tiny_problem(5, B=4, K=4, d=8, V=29)
    kw = dict(beta=1.0)
    B, K = 4, 4
    if case == "conf_one":
        kw["conf_in"] = np.ones(16)
    elif case == "k_one":
        B, K = 16, 1
    elif case == "decay_gamma_one":
        kw.update(mode=O.W_DECAY, gamma=1.0)
    else:
        kw.update(mode=O.W_UNIFORM)
    r = O.cat_loss_and_grads(H, W, y, B, K, **kw)
    assert abs(r["loss"] - _mean_nll(H, W, y)) < 1e-13
    assert np.all(r["w"] == 1.0)
    # gradient of the mean NLL by torch autograd (library pin)
    torch = pytest.importorskip("torch")
    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(y)).backward()
    np.testing.assert_allclose(r["dH"], Ht.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(r["dW"], Wt.grad.numpy(), atol=1e-14)


def test_beta_scales_linearly_and_sum_reduction():
    H, W, y = tiny_problem(6)
    conf = np.random.default_rng(6).random(12)
    a = O.cat_loss_and_grads(H, W, y, 3, 4, conf_in=conf, beta=1.0)
    b = O.cat_loss_and_grads(H, W, y, 3, 4, conf_in=conf, beta=0.1)
    c = O.cat_loss_and_grads(H, W, y, 3, 4, conf_in=conf, beta=1.0, reduction=O.RED_SUM)
    assert abs(b["loss"] - 0.1 * a["loss"]) < 1e-15
    np.testing.assert_allclose(b["dW"], 0.1 * a["dW"], rtol=1e-13, atol=1e-18)
    assert abs(c["loss"] - 12 * a["loss"]) < 1e-12
    np.testing.assert_allclose(c["dH"], 12 * a["dH"], rtol=1e-12, atol=1e-18)
    # Eq.11 per block: -(1/K) sum_k s_k log q_k, then averaged over the anchors
    per_block = [-(1 / 4) * np.sum(a["s"][i * 4:(i + 1) * 4] * a["logq"][i * 4:(i + 1) * 4]) for i in range(3)]
    assert abs(a["loss"] - np.mean(per_block)) < 1e-14


def test_weighted_ce_vs_torch_autograd_external_conf():
    """Eq.11 with constant weights: loss and grads equal torch's autograd of
    sum_t w_t * nll_t / N with w detached."""
    torch = pytest.importorskip("torch")
    H, W, y = tiny_problem(7, B=3, K=5, d=7, V=23)
    conf = np.random.default_rng(7).random(15)
    r = O.cat_loss_and_grads(H, W, y, 3, 5, conf_in=conf, beta=0.1)
    s = np.concatenate([np.cumprod(np.concatenate([[1.0], c[:-1]])) for c in conf.reshape(3, 5)])
    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    nll = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(y), reduction="none")
    loss = 0.1 * (torch.tensor(s) * nll).sum() / 15
    loss.backward()
    assert abs(r["loss"] - loss.item()) < 1e-14
    np.testing.assert_allclose(r["dH"], Ht.grad.numpy(), atol=1e-15)
    np.testing.assert_allclose(r["dW"], Wt.grad.numpy(), atol=1e-15)


# ------------------------------------------------------------ finite differences
def _loss_frozen(H, W, y, B, K, w, beta, n_valid):
    logq = log_softmax(H @ W.T, axis=1)[np.arange(len(y)), y]
    return beta / n_valid * np.sum(w * -logq)


@pytest.mark.parametrize("self_teacher", [False, True])
def test_finite_differences_with_frozen_weight(self_teacher):
    B, K, d, V = 2, 4, 5, 13
    H, W, y = tiny_problem(8, B, K, d, V)
    conf = None if self_teacher else np.random.default_rng(8).random(B * K)
    r = O.cat_loss_and_grads(H, W, y, B, K, conf_in=conf, beta=0.7)
    w = r["w"]
    eps = 1e-6
    rng = np.random.default_rng(80)
    for _ in range(12):
        t, i, v = rng.integers(B * K), rng.integers(d), rng.integers(V)
        Hp, Hm = H.copy(), H.copy()
        Hp[t, i] += eps
        Hm[t, i] -= eps
        fd = (_loss_frozen(Hp, W, y, B, K, w, 0.7, 8) - _loss_frozen(Hm, W, y, B, K, w, 0.7, 8)) / (2 * eps)
        assert abs(fd - r["dH"][t, i]) < 1e-7 * max(1, abs(fd)) + 1e-9
        Wp, Wm = W.copy(), W.copy()
        Wp[v, i] += eps
        Wm[v, i] -= eps
        fd = (_loss_frozen(H, Wp, y, B, K, w, 0.7, 8) - _loss_frozen(H, Wm, y, B, K, w, 0.7, 8)) / (2 * eps)
        assert abs(fd - r["dW"][v, i]) < 1e-7 * max(1, abs(fd)) + 1e-9


def test_self_teacher_weight_is_detached():
    """Stop-gradient (text before Eq.11): differentiating *through* the self-teacher
    weight gives a different derivative than the oracle's, which holds it constant."""
    B, K, d, V = 2, 4, 5, 13
    H, W, y = tiny_problem(9, B, K, d, V)
    r = O.cat_loss_and_grads(H, W, y, B, K, beta=1.0)
    eps = 1e-6
    # perturbing slot 0 of block 0 changes the weights of slots 1.. if not frozen
    Hp, Hm = H.copy(), H.copy()
    Hp[0, 0] += eps
    Hm[0, 0] -= eps
    lp = O.cat_forward(Hp, W, y, B, K)["loss"]
    lm = O.cat_forward(Hm, W, y, B, K)["loss"]
    fd_through = (lp - lm) / (2 * eps)
    assert abs(fd_through - r["dH"][0, 0]) > 1e-4 * abs(r["dH"][0, 0])


def test_gradient_invariants():
    H, W, y = tiny_problem(10, B=4, K=4, d=6, V=19)
    r = O.cat_loss_and_grads(H, W, y, 4, 4, beta=0.3)
    # sum_v dZ[t,v] = 0  =>  every column of dW sums to zero over the vocabulary
    np.testing.assert_allclose(r["dW"].sum(axis=0), 0, atol=1e-15)
    # <dW, W> = <dH, H>  (both equal sum_t g_t (sum_v q z - z_y))
    assert abs(np.sum(r["dW"] * W) - np.sum(r["dH"] * H)) < 1e-14


def test_sampled_backward_matches_full():
    H, W, y = tiny_problem(11, B=4, K=4, d=6, V=19)
    r = O.cat_loss_and_grads(H, W, y, 4, 4, beta=0.3)
    s = O.cat_backward(H, W, y, r["lse"], r["g"], rows=[3, 0, 9], vrows=[18, 2, y[0]])
    np.testing.assert_allclose(s["dH"], r["dH"][[3, 0, 9]], atol=1e-16)
    np.testing.assert_allclose(s["dW"], r["dW"][[18, 2, y[0]]], atol=1e-16)


# ---------------------------------------------------- masks, prefixes, edge cases
def test_accept_len_bruteforce():
    rng = np.random.default_rng(12)
    B, K = 50, 6
    hit = rng.random((B, K)) < 0.7
    vl = rng.integers(0, K + 1, B)
    got = O.accepted_prefix(hit.reshape(-1), B, K, vl)
    for b in range(B):
        best = 0
        for L in range(0, vl[b] + 1):
            if all(hit[b, :L]):
                best = L
        assert got[b] == best
    assert list(O.accepted_prefix(np.ones(6, bool), 1, 6)) == [6]
    assert list(O.accepted_prefix([False, True, True], 1, 3)) == [0]


def test_ignored_slots_and_valid_len():
    B, K, d, V = 2, 4, 5, 13
    H, W, y = tiny_problem(13, B, K, d, V)
    y = y.copy()
    y[2] = -100                                 # dropped slot inside block 0
    vl = np.array([4, 2])                       # block 1 keeps two slots
    r = O.cat_loss_and_grads(H, W, y, B, K, valid_len=vl, beta=1.0)
    assert r["n_valid"] == 3 + 2
    assert r["w"][2] == 0 and np.all(r["w"][6:] == 0)
    np.testing.assert_allclose(r["dH"][[2, 6, 7]], 0, atol=0)
    # self-teacher: the product runs through the dropped slot with c = 1
    assert r["s"][3] == r["s"][2]
    # the loss is the valid-mean of w * nll
    assert abs(r["loss"] - np.sum(r["w"] * -r["logq"]) / 5) < 1e-15
    # tail padding by ignore_index alone gives the same loss and grads as valid_len
    y2 = y.copy()
    y2[6:] = -100
    r2 = O.cat_loss_and_grads(H, W, y2, B, K, beta=1.0)
    assert abs(r2["loss"] - r["loss"]) < 1e-15
    np.testing.assert_allclose(r2["dW"], r["dW"], atol=1e-16)


def test_all_ignored_gives_zero():
    H, W, y = tiny_problem(14, 1, 4, 5, 9)
    r = O.cat_loss_and_grads(H, W, np.full(4, -100), 1, 4)
    assert r["loss"] == 0.0 and r["n_valid"] == 0
    assert not np.any(r["dH"]) and not np.any(r["dW"])


def test_out_of_range_target_raises():
    H, W, y = tiny_problem(15, 1, 4, 5, 9)
    with pytest.raises(ValueError):
        O.head_stats(H, W, [0, 9, 1, 2])


def test_target_logq_matches_head_stats():
    H, W, y = tiny_problem(16, B=3, K=4, d=6, V=21)
    y = y.copy()
    y[5] = -100
    st = O.head_stats(H, W, y)
    lq = O.target_logq(H, W.astype(np.float64), y, st["lse"])
    np.testing.assert_allclose(lq, st["logq"], atol=1e-14)
    Z = np.einsum("ti,vi->tv", H, W)
    ok = y >= 0
    np.testing.assert_allclose(lq[ok], log_softmax(Z, axis=1)[np.arange(12)[ok], y[ok]], atol=1e-13)


# ------------------------------------------------- anchor-dependent weights (Sec.3.3, Eq.12)
def test_weights_seq_hand_example_and_boundary():
    c = np.array([0.9, 0.5, 0.8, 0.25, 0.6])           # one sequence of N = 5 positions
    K = 3
    conf, vl, s, e = O.cat_weights_seq(c, anchor_pos=[0, 1, 2, 3, 4], seq_end=[5] * 5, K=K)
    assert list(vl) == [3, 3, 3, 2, 1]                    # slot k exists iff n + k <= N - 1
    np.testing.assert_allclose(s.reshape(5, K)[0], [1, 0.9, 0.45], atol=1e-15)
    np.testing.assert_allclose(s.reshape(5, K)[3][:2], [1, 0.25], atol=1e-15)
    np.testing.assert_allclose(conf.reshape(5, K)[3], [0.25, 0.6, 1.0], atol=0)
    assert abs(e[0] - (0.9 + 0.45 + 0.36)) < 1e-15 and abs(e[4] - 0.6) < 1e-15
    # Eq.12: for offset k the sum runs over N - k anchors
    for k in range(K):
        assert int((vl > k).sum()) == 5 - k


def test_weights_seq_sliding_identity_and_token_major_equivalence():
    rng = np.random.default_rng(17)
    N, K = 40, 6
    c = rng.random(N)
    anchors = np.arange(N)
    conf, vl, s, e = O.cat_weights_seq(c, anchors, np.full(N, N), K)
    S = s.reshape(N, K)
    for n in range(N - 1):
        for k in range(1, K):
            if n + k < N:                                  # s_{n,k} = c_n * s_{n+1,k-1}
                assert abs(S[n, k] - c[n] * S[n + 1, k - 1]) < 1e-15
    # same numbers as the token-major scan of Eq.10 on the gathered confidences
    s2, e2 = O.cat_weights(conf, N, K, valid_len=vl)
    np.testing.assert_allclose(s, s2, atol=1e-15)
    np.testing.assert_allclose(e, e2, atol=1e-14)
    # two sequences back to back: a block never reads across its own sequence's end
    conf3, vl3, _, _ = O.cat_weights_seq(c, [18, 19, 20], [20, 20, 40], K)
    assert list(vl3) == [2, 1, 6] and conf3.reshape(3, K)[0][2] == 1.0
    assert list(O.cat_weights_seq(c, [-1, 39], [40, 40], K)[1]) == [0, 1]
