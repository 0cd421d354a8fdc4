"""The contrast of the paper's pilot study (Section 2: the random-projection update rule that ends
the derivation, run with one fixed projection, against the same rule with a projection resampled
at every step; paragraph "Resampling random projection matrices": a fixed projection confines
the total change of W to a rank-r subspace, resampling lifts that), re-created on a generated
least-squares task instead of the paper's image data:

    loss(W) = 1/2 ||W - W*||_F^2,  gradient G = W - W*,  W <- W - eta (G A) A^T,  W_0 = 0.

With one projection for all steps every update lies in the row space of A^T, so W_t has rank
<= r and converges to the closed form W* A (A^T A)^-1 A^T; with a new projection per step
E[A A^T] = I makes the iteration contract towards W* itself and W_t becomes full rank.

The CPU part pins the oracle to those closed forms; the GPU part runs the same two schedules
through the C ABI (compress with a = 0, b = 1, then the SGD update) and checks the result both
against the oracle's trajectory and for the behaviour itself.
"""
import numpy as np
import pytest

import oracle


def run_oracle(Wstar, r, eta, steps, resample, gseed=3):
    n, m = Wstar.shape
    W = np.zeros((n, m))
    for t in range(steps):
        seed = oracle.derive_seed(gseed, 0, t if resample else 0)
        G = W - Wstar
        C = oracle.compress(G, r, seed)                      # G A
        W = oracle.sgd(W, oracle.decompress(C, m, seed), eta)  # W - eta (G A) A^T
    return W


def numerical_rank(W, rel=1e-6):
    s = np.linalg.svd(W, compute_uv=False)
    return int((s > rel * s[0]).sum()), s


def test_fixed_projection_is_confined_and_resampling_is_not():
    rng = np.random.default_rng(7)
    n, m, r, eta, steps = 24, 32, 4, 0.05, 300
    Wstar = rng.standard_normal((n, m))
    W_rp = run_oracle(Wstar, r, eta, steps, resample=False)
    W_rrp = run_oracle(Wstar, r, eta, steps, resample=True)
    # fixed projection: rank r, and the limit is the projection of W* onto the span of A
    rk, s = numerical_rank(W_rp, rel=1e-9)
    assert rk == r, s[:r + 2]
    A = oracle.materialise_A(oracle.derive_seed(3, 0, 0), m, r)
    P = A @ np.linalg.solve(A.T @ A, A.T)
    np.testing.assert_allclose(W_rp, Wstar @ P, rtol=0, atol=1e-9)
    # its loss cannot go below the part of W* outside that span
    floor = 0.5 * np.linalg.norm(Wstar @ (np.eye(m) - P)) ** 2
    loss_rp = 0.5 * np.linalg.norm(W_rp - Wstar) ** 2
    assert loss_rp == pytest.approx(floor, rel=1e-9)
    assert floor > 0.5 * 0.5 * np.linalg.norm(Wstar) ** 2          # r/m = 1/8 of the directions
    # resampled: full rank, and the loss falls by the expected factor per step,
    # 1 - 2 eta + eta^2 (m + r + 1) / r (second moment of A A^T), to within sampling noise
    rk, _ = numerical_rank(W_rrp)
    assert rk == min(n, m)
    loss_rrp = 0.5 * np.linalg.norm(W_rrp - Wstar) ** 2
    per_step = 1 - 2 * eta + eta * eta * (m + r + 1) / r
    expected = 0.5 * np.linalg.norm(Wstar) ** 2 * per_step ** steps
    assert loss_rrp < 1e-6 * loss_rp
    assert 1e-3 < loss_rrp / expected < 1e3                          # 300 steps of a random contraction


@pytest.mark.gpu
@pytest.mark.parametrize("r,bf16", [(8, False), (64, True)])
def test_contrast_through_the_library(r, bf16):
    torch = pytest.importorskip("torch")
    from paper_2402_03293_amd import flora
    dev = "cuda:0"
    # eta below 2 / lambda_max(A A^T), lambda_max about (sqrt(m) + sqrt(r))^2 / r
    n, m, eta, steps, gseed = 96, 320, 0.02 if r == 8 else 0.1, 120, 3
    g = torch.Generator(device="cpu").manual_seed(5)
    Wstar = torch.randn(n, m, generator=g)
    if bf16:
        Wstar = Wstar.to(torch.bfloat16).to(torch.float32)
    Wstar = Wstar.to(dev)
    tol = 1e-5 if r <= 32 else 2e-2
    out = {}
    for resample in (False, True):
        W = torch.zeros((n, m), device=dev)
        C = torch.zeros((n, r), device=dev)
        for t in range(steps):
            seed = flora.derive_seed(gseed, 0, t if resample else 0)
            G = W - Wstar                                    # the task's gradient (the model's side)
            if bf16:
                G = G.to(torch.bfloat16)
            mats = flora.matrices([(n, m)], grads=[G.contiguous()], weights=[W], states=[C], seeds=[seed])
            flora.fused_step(mats, r, flora.BF16 if bf16 else flora.F32, flora.F32, 0.0, 1.0, False,
                             flora.sgd_update(eta, 1.0))
        torch.cuda.synchronize()
        out[resample] = W.double().cpu().numpy()
    Ws = Wstar.double().cpu().numpy()
    # behaviour: confined to rank r with one projection, full rank and far lower loss when resampled
    s = np.linalg.svd(out[False], compute_uv=False)
    assert s[r] < (1e-5 if not bf16 else 2e-2) * s[0], s[:r + 2]
    s2 = np.linalg.svd(out[True], compute_uv=False)
    assert (s2 > 1e-3 * s2[0]).sum() == min(n, m)
    loss = {k: 0.5 * np.linalg.norm(v - Ws) ** 2 for k, v in out.items()}
    assert loss[True] < 0.2 * loss[False]
    if not bf16:
        # and the oracle's own trajectories (fp64 gradients of its own weights) end in the same place
        ref_rp = run_oracle(Ws, r, eta, steps, False, gseed)
        ref_rrp = run_oracle(Ws, r, eta, steps, True, gseed)
        e_rp = np.linalg.norm(out[False] - ref_rp) / np.linalg.norm(ref_rp)
        e_rrp = np.linalg.norm(out[True] - ref_rrp) / np.linalg.norm(ref_rrp)
        print("pilot contrast through the library: trajectory ends %.2e (fixed), %.2e (resampled) from the oracle's"
              % (e_rp, e_rrp))
        assert e_rp < tol and e_rrp < tol
    else:
        # bf16 gradients are rounded each step, which the fp64 trajectory does not model: compare
        # with the closed-form limit of the fixed projection instead (reached to rounding level)
        A = oracle.materialise_A(flora.derive_seed(gseed, 0, 0), m, r)
        P = A @ np.linalg.solve(A.T @ A, A.T)
        assert np.linalg.norm(out[False] - Ws @ P) / np.linalg.norm(Ws @ P) < tol
