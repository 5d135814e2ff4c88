"""Two-head HIP path (weighted beta CE + KD loss, Eq.12 under the forward-KL reading) vs its
fp64 oracle, element by element, through the C ABI.  Sizes the oracle finishes in seconds,
spanning several 128 x 256 tiles with ragged tails in every dimension; the teacher's width
differs from the draft's.

Tolerances as for the CE-only path (tests/helpers.py); KL(p || q) = a/s - lse_t + lse is a sum
of three terms each carrying the bf16 path's statistics error, so it gets 3x that tolerance.
"""
import numpy as np
import pytest

from oracle import cat_kd_oracle as KD
from oracle import cat_oracle as O
from paper_2605_08632_amd import synth
from tests import helpers as Hh

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _binding():
    from paper_2605_08632_amd import binding
    return binding


def _bf16_dev(bits, device="cuda:0"):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(device)


def _teacher_dev(p, device="cuda:0"):
    if p.dtype == "bf16":
        return _bf16_dev(p.teacher.H_bits, device), _bf16_dev(p.teacher.W_bits, device)
    return torch.from_numpy(p.teacher.H).to(device), torch.from_numpy(p.teacher.W).to(device)


def build_kd_problem(B, K, d, dt, V, seed, teacher="extend", dtype="bf16", **kw):
    p = Hh.build_problem(B, K, d, V, dtype, seed, **kw)
    p.teacher = p.head if teacher == "same" else synth.make_teacher(seed, p.head, dt)
    p.dt = p.teacher.H.shape[1]
    p.kd_stats = KD.kd_stats(p.head.H, p.W64, p.teacher.H, p.teacher.W.astype(np.float64), p.y)
    return p


def run_kd_case(p, beta=0.1, mode=O.W_CAT, gamma=1.0, reduction=O.RED_MEAN_VALID, external=False, grad_loss=None,
                accumulate=False):
    b = _binding()
    H, W, y, vl, conf = Hh.to_device(p)
    Ht, Wt = _teacher_dev(p)
    desc = b.make_desc(p.T, p.d, p.V, p.B, p.K, b.PARD2_BF16 if p.dtype == "bf16" else b.PARD2_FP32,
                       weight_mode=mode, reduction=reduction, beta=beta, gamma=gamma)
    ws = b.alloc_kd_workspace(desc, p.dt, H.device)
    beta32, gamma32 = float(np.float32(beta)), float(np.float32(gamma))
    ref = KD.cat_kd_forward(p.head.H, None, p.teacher.H, None, p.y, p.B, p.K,
                            conf_in=p.conf_ext if external else None, valid_len=p.valid_len, mode=mode, gamma=gamma32,
                            beta=beta32, reduction=reduction, stats=p.kd_stats)
    out = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, conf_in=conf if external else None, valid_len=vl, workspace=ws)
    torch.cuda.synchronize()
    g = Hh.check_forward(out, ref, p, stats_only=True)
    tol = Hh.TOL[p.dtype]
    np.testing.assert_allclose(g["lse_t"], ref["lse_t"], rtol=tol["stat"], atol=tol["stat"])
    np.testing.assert_allclose(g["kd"], ref["kd"], rtol=3 * tol["stat"], atol=3 * tol["stat"])
    np.testing.assert_allclose(g["w"], ref["w"], rtol=10 * tol["stat"], atol=1e-30)
    assert abs(g["loss"][0] - ref["loss"]) <= tol["loss"] * abs(ref["loss"]) + 1e-9, (g["loss"][0], ref["loss"])

    gout = 1.0 if grad_loss is None else grad_loss
    gr = KD.kd_row_scale(ref["w"], ref["n_valid"], reduction, gout)
    rb = KD.cat_kd_backward(p.head.H, p.W64, p.teacher.H, p.teacher.W, p.y, ref["lse"], ref["lse_t"], gr, beta32)
    gl = None if grad_loss is None else torch.tensor([grad_loss], dtype=torch.float32, device=H.device)
    dW0 = None
    if accumulate:
        dW0 = torch.from_numpy(np.random.default_rng(5).standard_normal((p.V, p.d)).astype(np.float32) *
                               np.float32(np.abs(rb["dW"]).max())).to(H.dtype).to(H.device)
    dH, dW = b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, out["lse"], out["lse_t"], out["w"], valid_len=vl, grad_loss=gl,
                                dW=None if dW0 is None else dW0.clone(), accumulate_dW=accumulate, workspace=ws)
    torch.cuda.synchronize()
    ref_dW = rb["dW"] if dW0 is None else rb["dW"] + dW0.float().cpu().numpy().astype(np.float64)
    eH, eW = Hh.check_grads(dH, dW, rb["dH"], ref_dW, p.dtype)
    inv = ~O.valid_mask(p.y, p.B, p.K, p.valid_len)
    if inv.any():
        assert not dH.float().cpu().numpy()[inv].any()

    # deferred loss: the forward without the cross term (two single-head sweeps), then a backward that also
    # returns KL per row and the loss from the logits it recomputes
    out2 = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, conf_in=conf if external else None, valid_len=vl, workspace=ws,
                              defer_loss=True)
    assert "loss" not in out2 and "kd" not in out2
    g2 = Hh.check_forward(out2, ref, p, stats_only=True)
    np.testing.assert_allclose(g2["lse_t"], ref["lse_t"], rtol=tol["stat"], atol=tol["stat"])
    np.testing.assert_allclose(g2["w"], ref["w"], rtol=10 * tol["stat"], atol=1e-30)
    kd2 = torch.empty(p.T, dtype=torch.float32, device=H.device)
    loss2 = torch.empty(1, dtype=torch.float32, device=H.device)
    dH2, dW2 = b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, out2["lse"], out2["lse_t"], out2["w"], valid_len=vl,
                                  grad_loss=gl, dW=None if dW0 is None else dW0.clone(), accumulate_dW=accumulate,
                                  workspace=ws, logp_y=out2["logp_y"], kd=kd2, loss=loss2)
    torch.cuda.synchronize()
    np.testing.assert_allclose(kd2.cpu().numpy(), ref["kd"], rtol=3 * tol["stat"], atol=3 * tol["stat"])
    assert abs(loss2.item() - ref["loss"]) <= tol["loss"] * abs(ref["loss"]) + 1e-9, (loss2.item(), ref["loss"])
    Hh.check_grads(dH2, dW2, rb["dH"], ref_dW, p.dtype)
    return eH, eW, out, (dH, dW)


@pytest.fixture(scope="module")
def kd_ragged():
    # T = 296 (one full 256-row tile + ragged), d = 200 and dt = 328 (k tails of 8), V = 1000
    # (eight 128-id tiles, the last ragged; the chunk's padded width holds one tile wholly past V)
    return build_kd_problem(37, 8, 200, 328, 1000, seed=31, ragged_frac=0.2, drop_some=True)


@pytest.mark.parametrize("variant", ["default", "beta1_sum", "external", "decay", "negative_gradloss", "accumulate"])
def test_kd_ragged(kd_ragged, variant):
    kw = {"default": dict(), "beta1_sum": dict(beta=1.0, reduction=O.RED_SUM), "external": dict(external=True),
          "decay": dict(mode=O.W_DECAY, gamma=0.8), "negative_gradloss": dict(grad_loss=-2.0),
          "accumulate": dict(accumulate=True)}[variant]
    run_kd_case(kd_ragged, **kw)


@pytest.mark.parametrize("variant", ["default", "beta1_sum_external", "accumulate_gradloss"])
def test_kd_fp32_storage(variant):
    """fp32 storage: plain fp32 FMA contractions, results track the fp64 definition to ~1e-6, so the
    two-head arithmetic is checked at 1e-5 instead of bf16's 1e-2.  Nothing divides the 64-wide tiles."""
    p = build_kd_problem(13, 5, 100, 148, 1001, seed=41, dtype="fp32", ragged_frac=0.3, drop_some=True)
    kw = {"default": dict(), "beta1_sum_external": dict(beta=1.0, reduction=O.RED_SUM, external=True),
          "accumulate_gradloss": dict(accumulate=True, grad_loss=-1.5)}[variant]
    run_kd_case(p, **kw)


def test_kd_multi_tile_k16():
    # several token tiles, vocabulary ranges of several tiles per workgroup, K = 16
    p = build_kd_problem(40, 16, 256, 512, 3000, seed=32, p_agree=("linear", 0.9, 0.3))
    run_kd_case(p)


def test_kd_odd_extents_and_narrow_teacher():
    # V one past a tile edge, T not a multiple of 8; teacher narrower than the draft (unrelated head)
    p = build_kd_problem(7, 5, 72, 40, 1025, seed=33, ragged_frac=0.3)
    run_kd_case(p, beta=0.5)
    p = build_kd_problem(3, 4, 32, 64, 127, seed=34)
    run_kd_case(p, beta=1.0)


def test_kd_teacher_equal_to_draft_matches_ce_only_path():
    """With the draft as its own teacher KD vanishes and the loss is the self-teacher CAT loss:
    the two-head kernels must then agree with the single-head ones (same library, other kernels)."""
    p = build_kd_problem(24, 8, 256, 256, 2000, seed=35, teacher="same")
    assert np.abs(p.kd_stats["kd"]).max() < 1e-12
    eH, eW, out, (dH, dW) = run_kd_case(p, beta=0.7)
    b = _binding()
    H, W, y, vl, _ = Hh.to_device(p)
    desc = b.make_desc(p.T, p.d, p.V, p.B, p.K, b.PARD2_BF16, beta=0.7)
    ce = b.pard2_cat_fwd(desc, H, W, y, valid_len=vl)
    dH2, dW2 = b.pard2_cat_bwd(desc, H, W, y, ce["lse"], ce["w"], valid_len=vl)
    torch.cuda.synchronize()
    assert torch.equal(out["argmax"], ce["argmax"]) and torch.equal(out["accept_len"], ce["accept_len"])
    np.testing.assert_allclose(out["loss"].cpu().numpy(), ce["loss"].cpu().numpy(), rtol=2e-3)
    assert np.abs(out["kd"].cpu().numpy()).max() < 3 * Hh.TOL["bf16"]["stat"]
    assert Hh.maxrel(dH.float().cpu().numpy(), dH2.float().cpu().numpy()) < 1e-2
    assert Hh.maxrel(dW.float().cpu().numpy(), dW2.float().cpu().numpy()) < 1e-2


def test_kd_medium_sampled():
    """T = 2048, d = 1024, dt = 2048, V = 32000: every forward output against the oracle; gradients on
    sampled token rows and vocabulary rows (the most frequent targets plus random ids)."""
    p = build_kd_problem(256, 8, 1024, 2048, 32000, seed=36, p_agree=0.6, fallback="zipf")
    b = _binding()
    H, W, y, vl, _ = Hh.to_device(p)
    Ht, Wt = _bf16_dev(p.teacher.H_bits), _bf16_dev(p.teacher.W_bits)
    desc = b.make_desc(p.T, p.d, p.V, p.B, p.K, b.PARD2_BF16, beta=0.1)
    ref = KD.cat_kd_forward(p.head.H, None, p.teacher.H, None, p.y, p.B, p.K, beta=float(np.float32(0.1)),
                            stats=p.kd_stats)
    out = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y)
    torch.cuda.synchronize()
    g = Hh.check_forward(out, ref, p, stats_only=True)
    tol = Hh.TOL["bf16"]
    np.testing.assert_allclose(g["kd"], ref["kd"], rtol=3 * tol["stat"], atol=3 * tol["stat"])
    assert abs(g["loss"][0] - ref["loss"]) <= tol["loss"] * abs(ref["loss"])
    dH, dW = b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, out["lse"], out["lse_t"], out["w"])
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(p.T, 96, replace=False))
    ids, cnt = np.unique(p.y, return_counts=True)
    vrows = np.unique(np.concatenate([ids[np.argsort(-cnt)[:64]], rng.choice(p.V, 192, replace=False)]))
    gr = KD.kd_row_scale(ref["w"], ref["n_valid"])
    rb = KD.cat_kd_backward(p.head.H, p.W64, p.teacher.H, p.teacher.W, p.y, ref["lse"], ref["lse_t"], gr,
                            float(np.float32(0.1)), rows=rows, vrows=vrows)
    # per-tensor scale: the full tensors' max magnitude is not known to the oracle here, so the sampled
    # rows' own max is the denominator (a stricter test)
    Hh.check_grads(dH, dW, rb["dH"], rb["dW"], "bf16", rows=rows, vrows=vrows)


def test_kd_minimum_sizes():
    for B, K, d, dt, V, seed in [(1, 1, 8, 16, 2, 61), (2, 3, 8, 8, 3, 62)]:
        run_kd_case(build_kd_problem(B, K, d, dt, V, seed=seed), beta=1.0)
