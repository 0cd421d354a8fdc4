"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
the whole matrix set of a workload goes through one grouped launch per call, and the
results are compared with the fp64 oracle on whole matrices where that takes seconds and on
sampled rows elsewhere.  Sampling rows is exact, not approximate: row i of the state and of
the decompressed gradient depends only on row i of G (Algorithm 1, compression and
decompression lines), and the transfer acts on each row of M with the same r x r matrix.
The factored update couples rows through its column statistics, so it is checked on whole
matrices, one of each shape.
"""
import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
from paper_2402_03293_amd import flora, workloads  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
from parity_bars import TOL_BF16, TOL_F32, update_bar  # noqa: E402


def to64(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_fro(x, ref):
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(np.asarray(x) - ref) / (den if den > 0 else 1.0))


def sample_rows(n, rng, blocks=(64, 128, 256, 512)):
    """First and last row, both sides of the row-block boundaries the kernels use, a few random."""
    rows = {0, n - 1}
    for b in blocks:
        for k in (1, 2):
            for d in (-1, 0):
                if 0 <= k * b + d < n:
                    rows.add(k * b + d)
    rows.update(int(x) for x in rng.integers(0, n, size=6))
    return np.array(sorted(rows))


def first_of_each_shape(shapes):
    seen, out = set(), []
    for l, s in enumerate(shapes):
        if s not in seen:
            seen.add(s)
            out.append(l)
    return out


@pytest.fixture(autouse=True)
def _free_gpu_memory():
    yield
    torch.cuda.empty_cache()


def test_workload2_full_cycle_every_matrix():
    """T5-small set, fp32, r = 16, tau = 8: all 96 matrices, every element."""
    wl = workloads.workload(2)
    r, tau, count = wl.r, wl.tau, len(wl.shapes)
    gen = workloads.make_generator(wl.seed, DEV)
    Gsets = [workloads.make_grad_set(wl, gen, DEV) for _ in range(tau)]
    W0 = workloads.make_weight_set(wl, gen, DEV)
    W = [w.clone() for w in W0]
    C = [torch.zeros((n, r), device=DEV) for n, _ in wl.shapes]
    gseed, epoch = 77, 3
    seeds = flora.derive_seeds(gseed, 0, count, epoch)
    for i in range(tau):
        flora.compress(flora.matrices(wl.shapes, grads=Gsets[i], states=C, seeds=seeds), r, flora.F32)
    torch.cuda.synchronize()
    Csnap = [c.clone() for c in C]
    flora.apply_update(flora.matrices(wl.shapes, weights=W, states=C, seeds=seeds), r, flora.F32,
                       flora.sgd_update(wl.lr, 1.0 / tau, zero_state_after=True))
    torch.cuda.synchronize()
    worst_c = worst_w = 0.0
    for l, (n, m) in enumerate(wl.shapes):
        seed = oracle.derive_seed(gseed, l, epoch)
        Cl = np.zeros((n, r))
        for i in range(tau):
            Cl = oracle.compress(to64(Gsets[i][l]), r, seed, state=Cl)
        Wl = oracle.sgd(to64(W0[l]), oracle.decompress(Cl, m, seed, alpha=1.0 / tau), wl.lr)
        worst_c = max(worst_c, rel_fro(to64(Csnap[l]), Cl))
        worst_w = max(worst_w, rel_fro(to64(W[l]) - to64(W0[l]), Wl - to64(W0[l])) / update_bar(r, Wl, to64(W0[l])))
        assert rel_fro(to64(W[l]), Wl) < 1e-6
        assert float(C[l].abs().max()) == 0.0
    print("workload 2: worst state err %.2e, worst update err %.2f of its bar" % (worst_c, worst_w))
    assert worst_c < TOL_F32
    assert worst_w < 1.0


def test_workload3_momentum_steps_with_transfer_sampled_rows():
    """GPT-2 base set, bf16, r = 64: three optimizer steps of Algorithm 2 through
    flora_fused_step with a resample at t = 0 and t = 2, whole set per launch."""
    _momentum_workload(workloads.workload(3), check=list(range(0, 48, 5)))


def test_workload5_fused_momentum_steps_sampled_rows():
    """GPT-2-XL set, bf16, r = 256, flora_fused_step on all 192 matrices."""
    wl = workloads.workload(5)
    _momentum_workload(wl, check=first_of_each_shape(wl.shapes) + [37, 102, 191])


def _momentum_workload(wl, check):
    r, count, beta, lr = wl.r, len(wl.shapes), wl.beta, wl.lr
    kappa, steps = 2, 3
    rng = np.random.default_rng(wl.index)
    gen = workloads.make_generator(wl.seed, DEV)
    Gsets = [workloads.make_grad_set(wl, gen, DEV) for _ in range(2)]
    W = workloads.make_weight_set(wl, gen, DEV)
    M = [torch.zeros((n, r), device=DEV) for n, _ in wl.shapes]
    rows = {l: sample_rows(wl.shapes[l][0], rng) for l in check}
    W_ref = {l: to64(W[l][torch.as_tensor(rows[l], device=DEV)]) for l in check}
    W_ini = {l: W_ref[l].copy() for l in check}
    M_ref = {l: np.zeros((len(rows[l]), r)) for l in check}
    gseed = 2024
    epoch = 0
    seeds = flora.derive_seeds(gseed, 0, count, epoch)
    upd = flora.sgd_update(lr, 1.0)
    for t in range(steps):
        G = Gsets[t % 2]
        resample = t % kappa == 0
        nxt = seeds
        if resample:
            epoch += 1
            nxt = flora.derive_seeds(gseed, 0, count, epoch)
        mats = flora.matrices(wl.shapes, grads=G, weights=W, states=M, seeds=seeds, seeds_next=nxt)
        flora.fused_step(mats, r, flora.BF16, flora.F32, beta, 1.0 - beta, resample, upd)
        torch.cuda.synchronize()
        for l in check:
            n, m = wl.shapes[l]
            s_old, s_new = int(seeds[l]), int(nxt[l])
            assert s_new == oracle.derive_seed(gseed, l, epoch)
            Mp = oracle.transfer(M_ref[l], m, s_old, s_new) if resample else M_ref[l]
            Grows = to64(G[l][torch.as_tensor(rows[l], device=DEV)])
            M_ref[l] = oracle.compress(Grows, r, s_new, state=Mp, a=beta, b=1.0 - beta)
            W_ref[l] = oracle.sgd(W_ref[l], oracle.decompress(M_ref[l], m, s_new), lr)
        seeds = nxt
    worst_m = worst_w = 0.0
    for l in check:
        idx = torch.as_tensor(rows[l], device=DEV)
        worst_m = max(worst_m, rel_fro(to64(M[l][idx]), M_ref[l]))
        worst_w = max(worst_w, rel_fro(to64(W[l][idx]) - W_ini[l], W_ref[l] - W_ini[l]))
    print("workload %d: worst state err %.2e, worst update err %.2e" % (wl.index, worst_m, worst_w))
    assert worst_m < TOL_BF16
    assert worst_w < TOL_BF16
    assert worst_m < 8e-3 and worst_w < 8e-3      # what bf16 operands should cost, with margin


def _momentum_schedule(wl, steps, kappa, check_rows, nring, checkpoints):
    """Algorithm 2 over `steps` optimizer steps with the projection resampled every `kappa`
    (t = 0 included), the whole matrix set in one flora_fused_step call per step, gradients
    cycling through a ring of `nring` sets.  `check_rows` maps a matrix index to the rows that are
    compared with oracle.Algorithm2 run on exactly those rows (a row of M, of the transfer and of
    the yield depends on no other row).  The checked matrices take the oracle driver's matrix ids
    0, 1, ... in its seed derivation; the others get ids of their own.  Returns the worst state
    and update errors over the checkpoints (steps after which both sides are compared)."""
    r, count, beta, lr = wl.r, len(wl.shapes), wl.beta, wl.lr
    gen = workloads.make_generator(wl.seed, DEV)
    ring = [workloads.make_grad_set(wl, gen, DEV) for _ in range(nring)]
    W = workloads.make_weight_set(wl, gen, DEV)
    M = [torch.zeros((n, r), device=DEV) for n, _ in wl.shapes]
    check = sorted(check_rows)
    idx = {l: torch.as_tensor(np.asarray(check_rows[l]), device=DEV) for l in check}
    gseed = 31337
    ids = np.arange(count, dtype=np.uint64) + 1000
    for c, l in enumerate(check):
        ids[l] = c

    def seeds_at(epoch):
        return np.array([flora.derive_seed(gseed, int(ids[l]), epoch) for l in range(count)], dtype=np.uint64)

    mats = [flora.matrices(wl.shapes, grads=ring[g], weights=W, states=M) for g in range(nring)]
    views = [flora.fields(mt) for mt in mats]
    upd = flora.sgd_update(lr, 1.0)
    W_ini = {l: to64(W[l][idx[l]]) for l in check}
    snaps = {}
    epoch, seeds = 0, seeds_at(0)
    for t in range(steps):
        resample = t % kappa == 0
        nxt = seeds
        if resample:
            epoch += 1
            nxt = seeds_at(epoch)
        v = views[t % nring]
        v["seed"][:] = seeds
        v["seed_next"][:] = nxt
        flora.fused_step(mats[t % nring], r, flora.BF16, flora.F32, beta, 1.0 - beta, resample, upd)
        seeds = nxt
        if t in checkpoints:
            snaps[t] = ({l: M[l][idx[l]].clone() for l in check}, {l: W[l][idx[l]].clone() for l in check})
    torch.cuda.synchronize()

    # the oracle's driver on the checked rows
    Grows = [[to64(ring[g][l][idx[l]]) for l in check] for g in range(nring)]
    orc = oracle.Algorithm2([(len(check_rows[l]), wl.shapes[l][1]) for l in check], r, beta, kappa, gseed)
    Wr = [W_ini[l].copy() for l in check]
    worst_m = worst_w = 0.0
    for t in range(steps):
        _, Wr = orc.step(Grows[t % nring], Wr, lr)
        if t in checkpoints:
            Ms, Ws = snaps[t]
            for c, l in enumerate(check):
                em = rel_fro(to64(Ms[l]), orc.M[c])
                ew = rel_fro(to64(Ws[l]) - W_ini[l], Wr[c] - W_ini[l])
                print("workload %d, matrix %d (%d x %d), after step %d: state err %.2e, update err %.2e"
                      % (wl.index, l, wl.shapes[l][0], wl.shapes[l][1], t, em, ew))
                worst_m, worst_w = max(worst_m, em), max(worst_w, ew)
    assert orc.transfers == len(check) * ((steps + kappa - 1) // kappa)
    return worst_m, worst_w


def test_workload3_whole_schedule_kappa100():
    """GPT-2 base set, bf16, r = 64, at the configuration's own schedule: 300 steps of Algorithm 2,
    beta = 0.9, projection resampled every 100 steps (the transfers at t = 100 and t = 200 act on a
    momentum that has run for a hundred steps), all 48 matrices per call.  One matrix of each of
    the four shapes is followed by the oracle: the 768 x 768 one whole, the others on sampled rows."""
    wl = workloads.workload(3)
    rng = np.random.default_rng(33)
    firsts = first_of_each_shape(wl.shapes)
    rows = {}
    for l in firsts:
        n, m = wl.shapes[l]
        rows[l] = np.arange(n) if n * m <= 768 * 768 else sample_rows(n, rng)
    wm, ww = _momentum_schedule(wl, steps=wl.steps, kappa=wl.kappa, check_rows=rows, nring=8,
                                checkpoints={0, 99, 100, 101, 200, 299})
    assert wm < TOL_BF16 and ww < TOL_BF16


def test_workload5_steps_with_a_transfer_in_the_middle():
    """GPT-2-XL set, bf16, r = 256: 24 steps of Algorithm 2 through flora_fused_step on all 192
    matrices, the projection resampled at t = 0 and t = 12; one matrix of each of the four shapes
    on sampled rows."""
    wl = workloads.workload(5)
    rng = np.random.default_rng(55)
    rows = {l: sample_rows(wl.shapes[l][0], rng) for l in first_of_each_shape(wl.shapes)}
    wm, ww = _momentum_schedule(wl, steps=24, kappa=12, check_rows=rows, nring=4, checkpoints={11, 12, 23})
    assert wm < TOL_BF16 and ww < TOL_BF16


def test_workload5_past_the_resample_at_step_1000():
    """GPT-2-XL set at the configuration's own resampling interval (kappa = 1000): 1003 steps on all
    192 matrices, so the transfer at t = 1000 moves a momentum that has accumulated for a thousand
    steps under bf16-rounded operands.  The oracle follows sixteen rows of the two shapes whose
    projection has 1600 rows (it rebuilds A on every call, which prices the wider ones out of a
    thousand steps; the 24-step test above covers those)."""
    wl = workloads.workload(5)
    rng = np.random.default_rng(56)
    rows = {}
    for l in first_of_each_shape(wl.shapes):
        n, m = wl.shapes[l]
        if m == 1600:
            rows[l] = np.sort(rng.choice(n, size=16, replace=False))
    assert len(rows) == 2
    wm, ww = _momentum_schedule(wl, steps=1003, kappa=wl.kappa, check_rows=rows, nring=4,
                                checkpoints={0, 500, 999, 1000, 1002})
    assert wm < TOL_BF16 and ww < TOL_BF16


def test_workload4_accumulate_and_factored_update():
    """T5-3B set, bf16, r = 256, tau = 16, factored update: all 384 matrices per launch; the
    accumulator is checked on sampled rows of several matrices, and the whole update (weights and
    both statistics) against the oracle on one whole matrix of each of the four shapes: the
    column statistics couple the rows, so the tall shape's 16 row blocks and the wide shape's 64
    column chunks are only covered by whole matrices."""
    wl = workloads.workload(4)
    r, tau, count = wl.r, wl.tau, len(wl.shapes)
    ex = wl.extra
    rng = np.random.default_rng(4)
    gen = workloads.make_generator(wl.seed, DEV)
    Gsets = [workloads.make_grad_set(wl, gen, DEV) for _ in range(2)]
    W = workloads.make_weight_set(wl, gen, DEV)
    C = [torch.zeros((n, r), device=DEV) for n, _ in wl.shapes]
    R = [torch.zeros((n,), device=DEV) for n, _ in wl.shapes]
    K = [torch.zeros((m,), device=DEV) for _, m in wl.shapes]
    gseed, epoch = 404, 1
    seeds = flora.derive_seeds(gseed, 0, count, epoch)
    firsts = first_of_each_shape(wl.shapes)                 # 1024x4096, 4096x1024, 1024x16384, 16384x1024
    whole = firsts
    sampled = firsts + [50, 200, 383]
    W0 = {l: to64(W[l]) for l in whole}
    rows = {l: sample_rows(wl.shapes[l][0], rng) for l in sampled}
    for i in range(tau):
        flora.compress(flora.matrices(wl.shapes, grads=Gsets[i % 2], states=C, seeds=seeds), r, flora.BF16)
    torch.cuda.synchronize()

    worst_c = 0.0
    for l in sampled:
        n, m = wl.shapes[l]
        idx = torch.as_tensor(rows[l], device=DEV)
        Cl = np.zeros((len(rows[l]), r))
        for i in range(tau):
            Cl = oracle.compress(to64(Gsets[i % 2][l][idx]), r, int(seeds[l]), state=Cl)
        worst_c = max(worst_c, rel_fro(to64(C[l][idx]), Cl))
    assert worst_c < TOL_BF16 and worst_c < 8e-3, worst_c

    # the oracle's own accumulators of the whole matrices (all tau micro-steps in fp64)
    # (the two 16M-element shapes: the cycle alternates between two gradients, and compression is
    # linear in G (Section 2.2; pinned on the CPU), so their sixteen compressions are taken as one
    # of G_0 + G_1 scaled by tau / 2 -- sixteen separate ones cost the oracle minutes)
    C_whole = {}
    for l in whole:
        n, m = wl.shapes[l]
        if n * m <= 1024 * 4096:
            Cl = np.zeros((n, r))
            for i in range(tau):
                Cl = oracle.compress(to64(Gsets[i % 2][l]), r, int(seeds[l]), state=Cl)
        else:
            Cl = oracle.compress(to64(Gsets[0][l]) + to64(Gsets[1][l]), r, int(seeds[l]), b=tau / 2.0)
        C_whole[l] = Cl
    upd = flora.factored_update(wl.lr, 1.0 / tau, ex["beta2"], ex["eps1"], ex["clip_d"], zero_state_after=True)
    flora.apply_update(flora.matrices(wl.shapes, weights=W, states=C, row_stats=R, col_stats=K, seeds=seeds),
                       r, flora.F32, upd)
    torch.cuda.synchronize()
    worst_u = worst_s = 0.0
    for l in whole:
        n, m = wl.shapes[l]
        Gt = oracle.decompress(C_whole[l], m, int(seeds[l]), alpha=1.0 / tau)
        Wr, Rr, Kr = oracle.factored_update(W0[l], Gt, np.zeros(n), np.zeros(m), ex["beta2"], ex["eps1"],
                                            ex["clip_d"], wl.lr)
        eu = rel_fro(to64(W[l]) - W0[l], Wr - W0[l])
        es = max(rel_fro(to64(R[l]), Rr), rel_fro(to64(K[l]), Kr))
        print("workload 4, %d x %d whole: statistics err %.2e, update err %.2e" % (n, m, es, eu))
        worst_u, worst_s = max(worst_u, eu), max(worst_s, es)
        del Gt, Wr
    print("workload 4: worst accumulator err %.2e, statistics err %.2e, update err %.2e"
          % (worst_c, worst_s, worst_u))
    assert worst_s < TOL_BF16 and worst_u < TOL_BF16
    for l in range(count):
        assert float(C[l].abs().max()) == 0.0
        assert bool(torch.isfinite(R[l]).all()) and bool(torch.isfinite(K[l]).all())
    # properties that hold at any size: sum_i R_i * m == sum_j K_j * n (both are the total of Q).
    # The two sides are computed independently (row sums through A^T A, column sums through S^T S,
    # each Gram matrix rounded to bf16 once), so they agree to that rounding averaged over the r
    # diagonal entries that carry the trace, about 2^-9 / sqrt(r), not to fp32 summation order
    for l in (100, 250, 383):
        n, m = wl.shapes[l]
        a, b = float(R[l].double().sum()) * m, float(K[l].double().sum()) * n
        assert abs(a - b) <= 1e-3 * abs(a)


@pytest.mark.parametrize("rule", ["adafactor", "unfactored"])
def test_workload4_shapes_whole_adafactor_step(rule):
    """T5-3B set, r = 256, all 384 matrices per launch, the whole Adafactor step (relative step,
    decay and parameter scale of the published schedules at step 7) with the factored or the
    unfactored second moment, from a seeded state and second moment.  Whole matrices of all
    four shapes against the oracle; the unfactored second moment (row by row independent) also on
    sampled rows of the last matrix, and the carried sum of squares everywhere."""
    wl = workloads.workload(4)
    r, count = wl.r, len(wl.shapes)
    rng = np.random.default_rng(44)
    gen = workloads.make_generator(wl.seed + 7, DEV)
    W = workloads.make_weight_set(wl, gen, DEV)
    S = [torch.randn((n, r), device=DEV, generator=gen) for n, _ in wl.shapes]
    seeds = flora.derive_seeds(414, 0, count, 3)
    firsts = first_of_each_shape(wl.shapes)
    whole = firsts
    large = [383]
    ss = torch.zeros((count, 4), device=DEV)
    sumsqs = [ss[l] for l in range(count)]
    kw = dict(weights=W, states=S, seeds=seeds, weight_sumsqs=sumsqs)
    R0 = K0 = V0 = None
    if rule == "adafactor":
        R = [torch.rand((n,), device=DEV, generator=gen) + 0.5 for n, _ in wl.shapes]
        K = [torch.rand((m,), device=DEV, generator=gen) + 0.5 for _, m in wl.shapes]
        R0 = {l: to64(R[l]) for l in whole}
        K0 = {l: to64(K[l]) for l in whole}
        kw.update(row_stats=R, col_stats=K)
    else:
        V = [torch.rand((n, m), device=DEV, generator=gen) + 0.5 for n, m in wl.shapes]
        rows = {l: sample_rows(wl.shapes[l][0], rng) for l in large}
        V0 = {l: to64(V[l]) for l in whole}
        V0.update({l: to64(V[l][torch.as_tensor(rows[l], device=DEV)]) for l in large})
        kw.update(second_moments=V)
    W0 = {l: to64(W[l]) for l in whole}
    S64 = {l: to64(S[l]) for l in whole}
    if rule == "unfactored":
        S64.update({l: to64(S[l][torch.as_tensor(rows[l], device=DEV)]) for l in large})
    mats = flora.matrices(wl.shapes, **kw)
    flora.weight_sumsq(mats)
    torch.cuda.synchronize()
    for l in (0, 100, 383):
        assert float(ss[l, 0]) == pytest.approx(float((W[l].double() ** 2).sum()), rel=5e-6)
    t, alpha, eps1, eps2, clip_d = 7, 1.0 / 16, 1e-30, 1e-3, 1.0
    rho, beta2 = flora.adafactor_schedule(t)
    mk = flora.factored_update if rule == "adafactor" else flora.unfactored_update
    flora.apply_update(mats, r, flora.F32, mk(rho, alpha, beta2, eps1, clip_d, scale_parameter=True, eps2=eps2))
    torch.cuda.synchronize()
    orho, obeta2 = oracle.adafactor_schedule(t)
    worst = 0.0
    for l in whole:
        n, m = wl.shapes[l]
        Gt = oracle.decompress(S64[l], m, int(seeds[l]), alpha=alpha)
        if rule == "adafactor":
            Wr, Rr, Kr = oracle.adafactor_step(W0[l], Gt, R=R0[l], K=K0[l], beta2=obeta2, eps1=eps1, eps2=eps2,
                                               clip_d=clip_d, step=orho)
            assert rel_fro(to64(R[l]), Rr) < TOL_BF16 and rel_fro(to64(K[l]), Kr) < TOL_BF16
        else:
            Wr, Vr = oracle.adafactor_step(W0[l], Gt, V=V0[l], beta2=obeta2, eps1=eps1, eps2=eps2, clip_d=clip_d,
                                           step=orho)
            assert rel_fro(to64(V[l]), Vr) < TOL_BF16
        worst = max(worst, rel_fro(to64(W[l]) - W0[l], Wr - W0[l]))
        assert float(ss[l, 0]) == pytest.approx(float((Wr ** 2).sum()), rel=1e-4)
    print("workload 4 shapes, %s: worst update err %.2e" % (rule, worst))
    assert worst < TOL_BF16
    if rule == "unfactored":
        for l in large:
            n, m = wl.shapes[l]
            Gt = oracle.decompress(S64[l], m, int(seeds[l]), alpha=alpha)
            Vr = obeta2 * V0[l] + (1.0 - obeta2) * (Gt * Gt + eps1)     # the elementwise EMA, rows independent
            got = to64(V[l][torch.as_tensor(rows[l], device=DEV)])
            assert rel_fro(got, Vr) < TOL_BF16
            assert (np.linalg.norm(got - Vr, axis=1) / np.linalg.norm(Vr, axis=1)).max() < TOL_BF16
    for l in range(0, count, 37):
        assert float(ss[l, 0]) == pytest.approx(float((W[l].double() ** 2).sum()), rel=5e-6)
        assert bool(torch.isfinite(W[l]).all())


@pytest.mark.parametrize("index", [2, 5])
def test_compressed_second_moment_at_full_size_sampled_rows(index):
    """flora_compress_mapped with the square map over a whole workload set in one grouped launch
    (fp32 path on workload 2, wide bf16 kernel with two rank slices on workload 5): two steps of the
    EMA, compared row by row with the oracle on sampled rows of a few matrices."""
    wl = workloads.workload(index)
    r, count = wl.r, len(wl.shapes)
    fd = flora.F32 if wl.grad_dtype == "f32" else flora.BF16
    rng = np.random.default_rng(100 + index)
    gen = workloads.make_generator(wl.seed, DEV)
    Gsets = [workloads.make_grad_set(wl, gen, DEV) for _ in range(2)]
    V = [torch.zeros((n, r), device=DEV) for n, _ in wl.shapes]
    seeds = flora.derive_seeds(77, 0, count, 0)
    beta2 = 0.8
    for t, G in enumerate(Gsets):
        mats = flora.matrices(wl.shapes, grads=G, states=V, seeds=seeds)
        flora.compress_mapped(mats, r, fd, flora.INPUT_SQUARE, 0.0 if t == 0 else beta2, 1.0 - beta2)
    torch.cuda.synchronize()
    check = first_of_each_shape(wl.shapes) + [count - 1]
    worst = 0.0
    for l in check:
        n, m = wl.shapes[l]
        rows = sample_rows(n, rng)
        idx = torch.as_tensor(rows, device=DEV)
        ref = np.zeros((len(rows), r))
        for t, G in enumerate(Gsets):
            ref = oracle.compress_mapped(to64(G[l][idx]), r, int(seeds[l]), "square", state=ref,
                                         a=0.0 if t == 0 else beta2, b=1.0 - beta2)
        got = to64(V[l][idx])
        per_row = np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)
        worst = max(worst, float(per_row.max()))
    print("workload %d: worst row err of the compressed second moment %.2e" % (index, worst))
    assert worst < (TOL_F32 if r <= 32 else TOL_BF16)
