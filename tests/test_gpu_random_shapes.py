"""Seeded sweep of random shapes and options through the same parity checks as the hand-picked
cases: B, K, d, V, storage type, beta, weight mode, reduction, external confidences, upstream
gradient, ragged blocks, dropped slots; every other case also runs the two-head (beta CE + KD) path
with a random teacher width."""
import numpy as np
import pytest

from tests import helpers as Hh
from tests import test_gpu_kd as K
from tests import test_gpu_parity as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("chunk", range(4))
def test_random_shapes(chunk):
    rng = np.random.default_rng([20260508, chunk])
    for it in range(8):
        dtype = "bf16" if rng.random() < 0.7 else "fp32"
        B = int(rng.integers(1, 70))
        Kk = int(rng.choice([1, 2, 4, 5, 8, 16]))
        d = int(rng.integers(1, 80)) * 8
        V = int(rng.integers(2, 5000))
        seed = int(rng.integers(1, 10 ** 6))
        kw = dict(beta=float(rng.choice([0.1, 0.5, 1.0])), mode=int(rng.choice([0, 0, 1, 2])),
                  gamma=float(rng.choice([1.0, 0.8])), reduction=int(rng.choice([0, 1])),
                  external=bool(rng.random() < 0.4), grad_loss=None if rng.random() < 0.5 else float(rng.normal() * 2))
        print(f"[random shapes] chunk {chunk} case {it}: {dtype} B={B} K={Kk} d={d} V={V} seed={seed} {kw}", flush=True)
        p = Hh.build_problem(B, Kk, d, V, dtype, seed=seed, p_agree=float(rng.choice([0.3, 0.6, 0.9])),
                             ragged_frac=float(rng.choice([0.0, 0.3])), drop_some=bool(rng.random() < 0.3))
        P._run_case(p, **kw)
        if it % 2 == 0:
            dt = int(rng.integers(1, 80)) * 8 if dtype == "bf16" else int(rng.integers(3, 300))
            q = K.build_kd_problem(B, Kk, d, dt, V, seed=seed, dtype=dtype, ragged_frac=float(rng.choice([0.0, 0.3])))
            K.run_kd_case(q, accumulate=bool(rng.random() < 0.3), **kw)
