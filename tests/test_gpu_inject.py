"""HIP gated target-feature injection (Sec.3.3) vs its fp64 oracle, element by element, through
the C ABI.  bf16 storage: outputs are rounded once from fp32 sums, so the bound is one bf16
rounding of the result (2^-8 relative) plus the fp32 accumulation error, taken per tensor.
"""
import numpy as np
import pytest

from oracle import inject_oracle as I
from paper_2605_08632_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _bf16(x):
    """numpy float32 -> (bf16-exact float64 copy, device bf16 tensor)"""
    bits = synth.f32_to_bf16_bits(x.astype(np.float32))
    exact = synth.bf16_bits_to_f32(bits).astype(np.float64)
    dev = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to("cuda:0")
    return exact, dev


def _case(seed, T, d, dt, F, rho=0.1, instance_rows=8):
    rng = np.random.default_rng(seed)
    E, Ed = _bf16(rng.standard_normal((T, d)))
    feats, featsd = zip(*[_bf16(rng.standard_normal((T, dt))) for _ in range(F)])
    P, Pd = _bf16(rng.standard_normal((d, F * dt)) / np.sqrt(F * dt))
    G, Gd = _bf16(rng.standard_normal((T, d)))
    # one Bernoulli(1 - rho) draw per training instance, repeated over the instance's rows
    n_inst = (T + instance_rows - 1) // instance_rows
    xi = np.repeat((rng.random(n_inst) >= rho).astype(np.float32), instance_rows)[:T]
    return E, Ed, list(feats), list(featsd), P, Pd, G, Gd, xi


def _close(gpu, ref, what):
    gpu = gpu.float().cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    err = np.abs(gpu - ref).max() / scale
    assert err <= 2.0 ** -8 + 1e-4, f"{what}: max error {err:.3e} of the tensor's scale"
    return err


@pytest.mark.parametrize("T,d,dt,F,rho", [
    (300, 264, 328, 3, 0.3),      # ragged in every dimension, k tails of 8
    (40, 64, 32, 1, 0.5),         # less than one tile, a single feature
    (1024, 512, 256, 4, 0.1),     # several tiles, four features (the paper's training set-up)
    (77, 520, 1032, 2, 0.0),      # T not a multiple of 8; rho = 0: always injected
])
def test_inject_parity(T, d, dt, F, rho):
    from paper_2605_08632_amd import binding as b
    E, Ed, feats, featsd, P, Pd, G, Gd, xi = _case(T * 7 + d, T, d, dt, F, rho)
    xid = torch.from_numpy(xi).to("cuda:0")
    ref = I.inject_forward(E, feats, P, xi)
    out = b.pard2_inject_fwd(Ed, featsd, Pd, xid)
    torch.cuda.synchronize()
    _close(out, ref, "Eout")
    gated_off = np.nonzero(xi == 0)[0]
    if len(gated_off):                                   # rows with the gate closed pass through bit-exactly
        assert torch.equal(out[torch.from_numpy(gated_off).to("cuda:0")], Ed[torch.from_numpy(gated_off).to("cuda:0")])
    rdT, rdP = I.inject_backward(G, feats, xi)
    dT, dP = b.pard2_inject_bwd(Gd, featsd, xid)
    torch.cuda.synchronize()
    assert np.array_equal(dT.float().cpu().numpy(), (xi[:, None] * G).astype(np.float32))   # 0/1 gate: exact
    _close(dP, rdP, "dP")
    # accumulate into an existing dP, and in-place forward
    dP0, dP0d = _bf16(np.random.default_rng(1).standard_normal(rdP.shape) * np.abs(rdP).max())
    _, dP2 = b.pard2_inject_bwd(Gd, featsd, xid, dP=dP0d.clone(), accumulate_dP=True)
    Ein = Ed.clone()
    b.pard2_inject_fwd(Ein, featsd, Pd, xid, Eout=Ein)
    torch.cuda.synchronize()
    _close(dP2, rdP + dP0, "dP +=")
    assert torch.equal(Ein, out)


def test_inject_fractional_gate_and_strided_features():
    from paper_2605_08632_amd import binding as b
    T, d, dt, F = 130, 72, 96, 3
    E, Ed, feats, featsd, P, Pd, G, Gd, _ = _case(5, T, d, dt, F)
    xi = np.random.default_rng(6).random(T).astype(np.float32)            # any real gate value is accepted
    # the three features as column blocks of one [T, 3*dt] tensor: row stride 3*dt
    big = torch.cat(featsd, dim=1).contiguous()
    views = [big[:, f * dt:(f + 1) * dt] for f in range(F)]
    xid = torch.from_numpy(xi).to("cuda:0")
    out = b.pard2_inject_fwd(Ed, views, Pd, xid)
    dT, dP = b.pard2_inject_bwd(Gd, views, xid)
    torch.cuda.synchronize()
    _close(out, I.inject_forward(E, feats, P, xi), "Eout")
    rdT, rdP = I.inject_backward(G, feats, xi)
    _close(dT, rdT, "dT")
    # dP is formed from the bf16-rounded dT: compare against the oracle run on that rounded operand too
    _close(dP, rdP, "dP")


def test_inject_large_shape_sampled():
    """T = 8192, d = 2048, F = 3 features of width 4096 (the 1B drafter under an 8B target): rows
    of Eout and rows of dP sampled, each computed one by one by the oracle."""
    from paper_2605_08632_amd import binding as b
    T, d, dt, F = 8192, 2048, 4096, 3
    g = torch.Generator(device="cuda:0")
    g.manual_seed(20260508)
    mk = lambda *s: torch.randn(*s, generator=g, device="cuda:0", dtype=torch.float32)
    Ed = mk(T, d).to(torch.bfloat16)
    featsd = [mk(T, dt).to(torch.bfloat16) for _ in range(F)]
    Pd = (mk(d, F * dt) / np.sqrt(F * dt)).to(torch.bfloat16)
    Gd = mk(T, d).to(torch.bfloat16)
    xi = np.repeat((np.random.default_rng(3).random(T // 512) >= 0.1).astype(np.float32), 512)
    xid = torch.from_numpy(xi).to("cuda:0")
    out = b.pard2_inject_fwd(Ed, featsd, Pd, xid)
    dT, dP = b.pard2_inject_bwd(Gd, featsd, xid)
    torch.cuda.synchronize()
    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    rows = np.array([0, 1, 255, 256, 511, 512, 4095, 4096, T - 2, T - 1])
    P64 = host(Pd)
    ref = I.inject_forward(host(Ed[rows]), [host(f[rows]) for f in featsd], P64, xi[rows])
    _close(out[rows], ref, "Eout rows")
    irows = np.array([0, 255, 256, 1023, d - 1])
    X = np.concatenate([host(f) for f in featsd], axis=1)
    ref_dP = (xi[:, None] * host(Gd)[:, irows]).T @ X
    _close(dP[irows], ref_dP, "dP rows")
