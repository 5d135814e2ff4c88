"""Full-size workloads (BASELINE configs 2-4) in the launch configuration bench.py times.

Forward: every row is compared with the oracle (argmax and accepted-prefix lengths bit-exact;
lse, log q(y), w, exp_len, loss within tolerance), using the oracle's stored target-independent
row statistics (tests/golden/fullsize_*.npz, written by make_fullsize_stats.py from oracle/ only).
Backward: dH on sampled whole blocks and dW on sampled vocabulary rows are computed one by one by
the oracle; in addition two identities that hold at any size are checked on the full tensors:
every column of dW sums to zero over the vocabulary, and <dW, W> = <dH, H>.
"""
import os

import numpy as np
import pytest

from oracle import cat_oracle as O
from paper_2605_08632_amd import synth
from tests import helpers as Hh

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("name", ["c2_llama1b_bf16", "c3_qwen06b_bf16", "c4_8bwidth_bf16"])
def test_fullsize_workload(name):
    from paper_2605_08632_amd import binding as b
    wl = synth.WORKLOADS[name]
    print(f"[fullsize] {name}: T={wl.T} d={wl.d} V={wl.V}", flush=True)
    stats = {k: v for k, v in np.load(os.path.join(GOLDEN, f"fullsize_{name}.npz")).items()}
    assert float(stats["gap_guard"]) == Hh.GAP_GUARD
    stats["argmax"] = stats["argmax"].astype(np.int64)
    p = Hh.build_problem(wl.B, wl.K, wl.d, wl.V, "bf16", wl.seed, p_agree=wl.p_agree, fallback=wl.fallback,
                         ragged_frac=wl.ragged_frac, stats=stats)
    H, W, y, vl, _ = Hh.to_device(p)
    desc = b.make_desc(p.T, p.d, p.V, p.B, p.K, b.PARD2_BF16, beta=wl.beta)
    beta = float(np.float32(wl.beta))
    ws = b.alloc_workspace(desc, H.device)

    # ---- forward: all rows
    ref = Hh.oracle_forward(p, beta=beta)
    out = b.pard2_cat_fwd(desc, H, W, y, valid_len=vl, workspace=ws)
    Hh.check_forward(out, ref, p)
    print(f"[fullsize] forward ok: loss {out['loss'].item():.6f} oracle {ref['loss']:.6f}, "
          f"{p.regenerated} near-tie rows re-drawn", flush=True)

    # ---- backward: sampled rows / vocabulary rows against the oracle
    dH, dW = b.pard2_cat_bwd(desc, H, W, y, out["lse"], out["w"], valid_len=vl, workspace=ws)
    torch.cuda.synchronize()
    g = O.row_scale(ref["w"], beta, ref["n_valid"])
    rng = np.random.default_rng([wl.seed, 77])
    blocks = {0, wl.B - 1, wl.B // 2}
    blocks |= set(rng.integers(0, wl.B, 5).tolist())
    if p.valid_len is not None:                       # make sure ragged blocks are sampled
        blocks |= set(np.nonzero(p.valid_len < wl.K)[0][:3].tolist())
    rows = np.concatenate([np.arange(bk * wl.K, (bk + 1) * wl.K) for bk in sorted(blocks)])
    ids, counts = np.unique(p.y[p.y >= 0], return_counts=True)
    frequent = ids[np.argsort(-counts)[:96]]
    edges = np.array([0, 255, 256, 16383, 16384, wl.V - 257, wl.V - 2, wl.V - 1])
    vrows = np.unique(np.concatenate([frequent, edges, rng.integers(0, wl.V, 96)]))
    rb = O.cat_backward(p.head.H, None, p.y, ref["lse"], g, rows=rows, vrows=vrows, W64=p.W64, slab=64)
    # normalise by the full tensors' scale: the sampled rows hold the largest entries (frequent ids)
    gH = dH[torch.from_numpy(rows).to(H.device)].float().cpu().numpy()
    gW = dW[torch.from_numpy(vrows).to(H.device)].float().cpu().numpy()
    eH = np.max(np.abs(gH - rb["dH"])) / np.max(np.abs(rb["dH"]))
    eW = np.max(np.abs(gW - rb["dW"])) / np.max(np.abs(rb["dW"]))
    print(f"[fullsize] backward sampled: dH max-rel {eH:.2e} ({len(rows)} rows), "
          f"dW max-rel {eW:.2e} ({len(vrows)} vocabulary rows)", flush=True)
    assert eH <= Hh.TOL["bf16"]["grad"] and eW <= Hh.TOL["bf16"]["grad"]
    inv = ~O.valid_mask(p.y, p.B, p.K, p.valid_len)
    if inv.any():
        assert not dH[torch.from_numpy(np.nonzero(inv)[0]).to(H.device)].float().any().item()

    # ---- identities on the full tensors (fp64 on the device: plumbing, not the method)
    dW64, dH64 = dW.double(), dH.double()
    colsum = dW64.sum(dim=0).abs()
    colabs = dW64.abs().sum(dim=0)
    assert (colsum <= 1e-3 * colabs + 1e-30).all().item(), "columns of dW do not sum to zero"
    lhs = (dW64 * W.double()).sum().item()
    rhs = (dH64 * H.double()).sum().item()
    assert abs(lhs - rhs) <= 1e-2 * max(abs(lhs), abs(rhs)), (lhs, rhs)
    print(f"[fullsize] identities ok: <dW,W> {lhs:.6e} <dH,H> {rhs:.6e}", flush=True)


@pytest.mark.parametrize("name,dt", [("c2_llama1b_bf16", 4096), ("c3_qwen06b_bf16", 4096)])
def test_fullsize_kd(name, dt):
    """The Eq.12 token loss (beta CE + KD) at full-size shapes with a teacher head of width 4096,
    in the launch configuration `bench.py --variant kd` times (the second workload's vocabulary is
    not a multiple of 256: its last chunk holds a 128-id tile that lies wholly past V).  Forward: every row against the oracle
    (the teacher's logsumexp and KL(p || q) of every row are stored by make_fullsize_stats.py, from
    oracle/ only).  Backward: sampled blocks / vocabulary rows one by one, plus the two identities."""
    from oracle import cat_kd_oracle as KD
    from paper_2605_08632_amd import binding as b
    wl = synth.WORKLOADS[name]
    print(f"[fullsize kd] {name}: T={wl.T} d={wl.d} dt={dt} V={wl.V}", flush=True)
    stats = {k: v for k, v in np.load(os.path.join(GOLDEN, f"fullsize_{name}.npz")).items()}
    stats["argmax"] = stats["argmax"].astype(np.int64)
    gold = np.load(os.path.join(GOLDEN, f"fullsize_kd_{name}_dt{dt}.npz"))
    assert int(gold["teacher_d"]) == dt
    p = Hh.build_problem(wl.B, wl.K, wl.d, wl.V, "bf16", wl.seed, p_agree=wl.p_agree, fallback=wl.fallback,
                         ragged_frac=wl.ragged_frac, stats=stats)
    teacher = synth.make_teacher(wl.seed, p.head, dt)
    kst = dict(p.stats)
    kst["lse_t"], kst["kd"] = gold["lse_t"], gold["kd"]
    kst["logp_t"] = O.target_logq(teacher.H, teacher.W, p.y, gold["lse_t"])
    beta = float(np.float32(wl.beta))
    ref = KD.cat_kd_forward(p.head.H, None, teacher.H, None, p.y, p.B, p.K, valid_len=p.valid_len, beta=beta,
                            stats=kst)

    H, W, y, vl, _ = Hh.to_device(p)
    Ht = torch.from_numpy(teacher.H_bits.view(np.int16)).view(torch.bfloat16).to(H.device)
    Wt = torch.from_numpy(teacher.W_bits.view(np.int16)).view(torch.bfloat16).to(H.device)
    desc = b.make_desc(p.T, p.d, p.V, p.B, p.K, b.PARD2_BF16, beta=wl.beta)
    ws = b.alloc_kd_workspace(desc, dt, H.device)
    out = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, valid_len=vl, workspace=ws)
    torch.cuda.synchronize()
    g = Hh.check_forward(out, ref, p, stats_only=True)
    tol = Hh.TOL["bf16"]
    np.testing.assert_allclose(g["lse_t"], ref["lse_t"], rtol=tol["stat"], atol=tol["stat"])
    np.testing.assert_allclose(g["kd"], ref["kd"], rtol=3 * tol["stat"], atol=3 * tol["stat"])
    np.testing.assert_allclose(g["w"], ref["w"], rtol=10 * tol["stat"], atol=1e-30)
    assert abs(g["loss"][0] - ref["loss"]) <= tol["loss"] * abs(ref["loss"])
    print(f"[fullsize kd] forward ok: loss {g['loss'][0]:.6f} oracle {ref['loss']:.6f}, "
          f"mean KL {ref['kd'].mean():.4f}", flush=True)

    dH, dW = b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, out["lse"], out["lse_t"], out["w"], valid_len=vl,
                                workspace=ws)
    torch.cuda.synchronize()
    gr = KD.kd_row_scale(ref["w"], ref["n_valid"])
    rng = np.random.default_rng([wl.seed, 78])
    blocks = {0, wl.B - 1, wl.B // 2} | set(rng.integers(0, wl.B, 5).tolist())
    rows = np.concatenate([np.arange(bk * wl.K, (bk + 1) * wl.K) for bk in sorted(blocks)])
    ids, counts = np.unique(p.y[p.y >= 0], return_counts=True)
    frequent = ids[np.argsort(-counts)[:96]]
    edges = np.array([0, 127, 128, 16383, 16384, wl.V - 129, wl.V - 2, wl.V - 1])
    vrows = np.unique(np.concatenate([frequent, edges, rng.integers(0, wl.V, 96)]))
    rb = KD.cat_kd_backward(p.head.H, p.W64, teacher.H, teacher.W, p.y, ref["lse"], ref["lse_t"], gr, beta,
                            slab=64, rows=rows, vrows=vrows)
    gH = dH[torch.from_numpy(rows).to(H.device)].float().cpu().numpy()
    gW = dW[torch.from_numpy(vrows).to(H.device)].float().cpu().numpy()
    eH = np.max(np.abs(gH - rb["dH"])) / np.max(np.abs(rb["dH"]))
    eW = np.max(np.abs(gW - rb["dW"])) / np.max(np.abs(rb["dW"]))
    print(f"[fullsize kd] backward sampled: dH max-rel {eH:.2e} ({len(rows)} rows), "
          f"dW max-rel {eW:.2e} ({len(vrows)} vocabulary rows)", flush=True)
    assert eH <= tol["grad"] and eW <= tol["grad"]

    dW64, dH64 = dW.double(), dH.double()
    colsum = dW64.sum(dim=0).abs()
    colabs = dW64.abs().sum(dim=0)
    assert (colsum <= 1e-3 * colabs + 1e-30).all().item(), "columns of dW do not sum to zero"
    lhs = (dW64 * W.double()).sum().item()
    rhs = (dH64 * H.double()).sum().item()
    assert abs(lhs - rhs) <= 1e-2 * max(abs(lhs), abs(rhs)), (lhs, rhs)
    print(f"[fullsize kd] identities ok: <dW,W> {lhs:.6e} <dH,H> {rhs:.6e}", flush=True)

    # deferred loss (the configuration `bench.py --variant kd-deferred` times): forward without the cross
    # term, KL per row and loss from the backward
    out2 = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, valid_len=vl, workspace=ws, defer_loss=True)
    kd2 = torch.empty(p.T, dtype=torch.float32, device=H.device)
    loss2 = torch.empty(1, dtype=torch.float32, device=H.device)
    dH2, dW2 = b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, out2["lse"], out2["lse_t"], out2["w"], valid_len=vl,
                                  workspace=ws, logp_y=out2["logp_y"], kd=kd2, loss=loss2)
    torch.cuda.synchronize()
    g2 = Hh.check_forward(out2, ref, p, stats_only=True)
    np.testing.assert_allclose(g2["lse_t"], ref["lse_t"], rtol=tol["stat"], atol=tol["stat"])
    np.testing.assert_allclose(kd2.cpu().numpy(), ref["kd"], rtol=3 * tol["stat"], atol=3 * tol["stat"])
    assert abs(loss2.item() - ref["loss"]) <= tol["loss"] * abs(ref["loss"])
    eH = np.max(np.abs(dH2[torch.from_numpy(rows).to(H.device)].float().cpu().numpy() - rb["dH"])) / np.max(np.abs(rb["dH"]))
    eW = np.max(np.abs(dW2[torch.from_numpy(vrows).to(H.device)].float().cpu().numpy() - rb["dW"])) / np.max(np.abs(rb["dW"]))
    assert eH <= tol["grad"] and eW <= tol["grad"]
    print(f"[fullsize kd] deferred loss ok: loss {loss2.item():.6f}, dH {eH:.2e}, dW {eW:.2e}", flush=True)
