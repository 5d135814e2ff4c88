"""The autograd front end against torch's OWN cross-entropy and KL on the GPU: in the cases where the
CAT loss reduces to a library routine (UNIFORM weights = plain mean cross-entropy, Eq.5; external
confidences = a weighted one) the HIP path is checked against an implementation that shares nothing
with it or with the oracle.  fp32 storage, so the comparison is tight."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
F = torch.nn.functional


def _inputs(seed, B, K, d, V, dt=None):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    T = B * K
    H = torch.randn(T, d, generator=g, device="cuda:0")
    W = torch.randn(V, d, generator=g, device="cuda:0") * (3.0 / d ** 0.5)
    y = torch.randint(0, V, (T,), generator=g, device="cuda:0", dtype=torch.int32)
    y[::7] = -100
    out = [H, W, y]
    if dt:
        out += [torch.randn(T, dt, generator=g, device="cuda:0"),
                torch.randn(V, dt, generator=g, device="cuda:0") * (3.0 / dt ** 0.5)]
    return out


def test_uniform_mode_equals_torch_cross_entropy():
    from paper_2605_08632_amd import autograd as A, binding as b
    H, W, y = _inputs(1, 12, 5, 96, 777)
    H1, W1 = H.clone().requires_grad_(), W.clone().requires_grad_()
    loss = A.cat_loss(H1, W1, y, 12, 5, weight_mode=b.PARD2_W_UNIFORM, beta=1.0)
    (2.5 * loss).backward()
    H2, W2 = H.clone().requires_grad_(), W.clone().requires_grad_()
    ref = F.cross_entropy(H2 @ W2.t(), y.long(), ignore_index=-100, reduction="mean")
    (2.5 * ref).backward()
    assert abs(loss.item() - ref.item()) < 1e-5 * abs(ref.item())
    assert (H1.grad - H2.grad).abs().max() < 1e-5 * H2.grad.abs().max()
    assert (W1.grad - W2.grad).abs().max() < 1e-5 * W2.grad.abs().max()


def test_external_confidences_equal_a_weighted_torch_cross_entropy():
    from paper_2605_08632_amd import autograd as A
    B, K = 9, 6
    H, W, y = _inputs(2, B, K, 64, 500)
    conf = torch.rand(B * K, device="cuda:0")
    H1, W1 = H.clone().requires_grad_(), W.clone().requires_grad_()
    loss = A.cat_loss(H1, W1, y, B, K, conf_in=conf, beta=0.3)
    loss.backward()
    # Eq.10 with torch: exclusive cumulative product per block
    c = conf.reshape(B, K)
    s = torch.cat([torch.ones(B, 1, device="cuda:0"), torch.cumprod(c, dim=1)[:, :-1]], dim=1).reshape(-1)
    H2, W2 = H.clone().requires_grad_(), W.clone().requires_grad_()
    nll = F.cross_entropy(H2 @ W2.t(), y.long(), ignore_index=-100, reduction="none")
    valid = y >= 0
    ref = 0.3 * (s * nll)[valid].sum() / valid.sum()
    ref.backward()
    assert abs(loss.item() - ref.item()) < 1e-5 * abs(ref.item())
    assert (H1.grad - H2.grad).abs().max() < 1e-5 * H2.grad.abs().max()
    assert (W1.grad - W2.grad).abs().max() < 1e-5 * W2.grad.abs().max()


def test_kd_loss_equals_torch_kl_div_plus_cross_entropy():
    from paper_2605_08632_amd import autograd as A, binding as b
    B, K = 8, 4
    H, W, y, Ht, Wt = _inputs(3, B, K, 72, 300, dt=104)
    H1, W1 = H.clone().requires_grad_(), W.clone().requires_grad_()
    loss = A.cat_kd_loss(H1, W1, Ht, Wt, y, B, K, weight_mode=b.PARD2_W_UNIFORM, beta=0.2)
    loss.backward()
    H2, W2 = H.clone().requires_grad_(), W.clone().requires_grad_()
    logq = F.log_softmax(H2 @ W2.t(), dim=1)
    kd = F.kl_div(logq, F.softmax(Ht @ Wt.t(), dim=1), reduction="none").sum(dim=1)
    nll = F.nll_loss(logq, y.long(), ignore_index=-100, reduction="none")
    valid = y >= 0
    ref = (0.2 * nll + kd)[valid].sum() / valid.sum()
    ref.backward()
    assert abs(loss.item() - ref.item()) < 2e-5 * abs(ref.item())
    assert (H1.grad - H2.grad).abs().max() < 2e-5 * H2.grad.abs().max()
    assert (W1.grad - W2.grad).abs().max() < 2e-5 * W2.grad.abs().max()


def test_bf16_storage_through_autograd():
    from paper_2605_08632_amd import autograd as A
    H, W, y = _inputs(4, 40, 8, 256, 3000)
    H1, W1 = H.bfloat16().requires_grad_(), W.bfloat16().requires_grad_()
    loss = A.cat_loss(H1, W1, y, 40, 8, beta=1.0)
    loss.backward()
    assert H1.grad.dtype == torch.bfloat16 and torch.isfinite(H1.grad.float()).all() and H1.grad.float().abs().sum() > 0
    assert W1.grad.shape == W1.shape
