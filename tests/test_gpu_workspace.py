"""Caller-owned workspace (flora_set_workspace): every entry point gives the same bits whether the
library allocates its private device memory itself or carves it from the caller's buffer; a
workspace that is too small is refused before anything runs; flora_workspace_bytes is exact; and
in workspace mode the device's free memory does not move."""
import ctypes

import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
from paper_2402_03293_amd import flora  # noqa: E402
from parity_bars import tol_for  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to64(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_fro(x, ref):
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(np.asarray(x) - ref) / (den if den > 0 else 1.0))


@pytest.fixture(autouse=True)
def _back_to_library_memory():
    yield
    torch.cuda.synchronize()
    flora.set_workspace(None)


def _inputs(shapes, r, bf16, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    gdt = torch.bfloat16 if bf16 else torch.float32
    return dict(
        G=[torch.randn(*s, generator=g).to(gdt).to(DEV) for s in shapes],
        W=[torch.randn(*s, generator=g).to(DEV) for s in shapes],
        M=[torch.randn(n, r, generator=g).to(DEV) for n, _ in shapes],
        R=[torch.rand(n, generator=g).to(DEV) + 0.5 for n, _ in shapes],
        K=[torch.rand(m, generator=g).to(DEV) + 0.5 for _, m in shapes],
    )


def _step_sequence(shapes, r, bf16, x):
    """A transfer + compress + SGD update (fused), then a factored update, a plain compress, a
    decompress and the sum of squares, on clones of x; returns everything that was written."""
    count = len(shapes)
    W = [w.clone() for w in x["W"]]
    M = [m.clone() for m in x["M"]]
    R = [v.clone() for v in x["R"]]
    K = [v.clone() for v in x["K"]]
    out = [torch.empty(s, device=DEV) for s in shapes]
    ss = torch.zeros((count, 4), device=DEV)
    s0 = [int(flora.derive_seed(5, l, 0)) for l in range(count)]
    s1 = [int(flora.derive_seed(5, l, 1)) for l in range(count)]
    fd = flora.BF16 if bf16 else flora.F32
    mats = flora.matrices(shapes, grads=x["G"], weights=W, states=M, row_stats=R, col_stats=K, seeds=s0, seeds_next=s1,
                          weight_sumsqs=[ss[l] for l in range(count)])
    flora.fused_step(mats, r, fd, flora.F32, 0.9, 0.1, True, flora.sgd_update(1e-2, 1.0))
    mats1 = flora.matrices(shapes, grads=x["G"], weights=W, states=M, row_stats=R, col_stats=K, seeds=s1,
                           weight_sumsqs=[ss[l] for l in range(count)])
    flora.weight_sumsq(mats1)
    flora.apply_update(mats1, r, flora.F32, flora.factored_update(1e-2, 0.5, 0.5, 1e-30, 1.0, scale_parameter=True))
    flora.compress(mats1, r, fd, 0.5, 2.0)
    flora.decompress(mats1, r, 0.25, out, flora.F32)
    torch.cuda.synchronize()
    return W + M + R + K + out + [ss]


@pytest.mark.parametrize("r,bf16,shapes", [
    (16, False, [(130, 200), (64, 2048), (300, 77)]),
    (64, True, [(300, 520), (256, 1536)]),
    (256, True, [(257, 264), (512, 2048), (128, 4096)]),
    (128, False, [(100, 136), (260, 1032)]),
])
def test_same_bits_with_and_without_a_caller_owned_workspace(r, bf16, shapes):
    x = _inputs(shapes, r, bf16, 100 + r)
    flora.set_workspace(None)
    ref = _step_sequence(shapes, r, bf16, x)
    need = flora.workspace_bytes(flora.matrices(shapes), r)
    # (a) roomy: every plan of the sequence stays resident
    ws = torch.empty(4 * need + (1 << 20), dtype=torch.uint8, device=DEV)
    flora.set_workspace(ws)
    got = _step_sequence(shapes, r, bf16, x)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    got = _step_sequence(shapes, r, bf16, x)          # second time: plans and images found again
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    # (b) exactly flora_workspace_bytes: the calls after the fused step push its plans out and refill
    torch.cuda.synchronize()
    ws2 = torch.empty(need, dtype=torch.uint8, device=DEV)
    flora.set_workspace(ws2)
    for _ in range(2):
        got = _step_sequence(shapes, r, bf16, x)
        for a, b in zip(ref, got):
            assert torch.equal(a, b)
    # and against the oracle, once (the first state of the sequence: transfer, then EMA compress)
    l = 0
    n, m = shapes[l]
    s0, s1 = int(flora.derive_seed(5, l, 0)), int(flora.derive_seed(5, l, 1))
    Mr = oracle.compress(to64(x["G"][l]), r, s1, state=oracle.transfer(to64(x["M"][l]), m, s0, s1), a=0.9, b=0.1)
    Mr = oracle.compress(to64(x["G"][l]), r, s1, state=Mr, a=0.5, b=2.0)
    assert rel_fro(to64(got[len(shapes) + l]), Mr) < tol_for(r)


def test_workspace_bytes_is_exact_and_too_small_changes_nothing():
    shapes, r = [(512, 2048), (300, 520)], 256
    x = _inputs(shapes, r, True, 7)
    count = len(shapes)
    need = flora.workspace_bytes(flora.matrices(shapes), r)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    W = [w.clone() for w in x["W"]]
    M = [m.clone() for m in x["M"]]
    R = [v.clone() for v in x["R"]]
    K = [v.clone() for v in x["K"]]
    mats = flora.matrices(shapes, grads=x["G"], weights=W, states=M, row_stats=R, col_stats=K,
                          seeds=[1] * count, seeds_next=[2] * count)
    fac = flora.factored_update(1e-2, 1.0, 0.0, 1e-30, 1.0)
    L = flora.lib()
    # one 256-byte unit short: refused, and nothing was enqueued
    flora.set_workspace(ws, need - 256)
    st = L.flora_fused_step(mats, count, r, flora.BF16, flora.F32, 0.9, 0.1, 1, ctypes.byref(fac), None)
    assert st == flora.ERR_INVALID
    torch.cuda.synchronize()
    for a, b in zip(W + M + R + K, x["W"] + x["M"] + x["R"] + x["K"]):
        assert torch.equal(a, b)
    # the smaller calls still fit
    flora.compress(mats, r, flora.BF16, 0.5, 0.5)
    torch.cuda.synchronize()
    assert not torch.equal(M[0], x["M"][0])
    # exactly the stated size: accepted
    flora.set_workspace(ws, need)
    st = L.flora_fused_step(mats, count, r, flora.BF16, flora.F32, 0.9, 0.1, 1, ctypes.byref(fac), None)
    assert st == flora.OK
    torch.cuda.synchronize()
    assert not torch.equal(W[0], x["W"][0])


def test_no_device_allocation_with_a_workspace():
    """With a workspace set, calls on shapes the library has never seen leave the device's free
    memory where it was (the library-allocated mode takes megabytes for the same calls)."""
    r, bf16 = 256, True
    first, second = [(384, 1280), (256, 2304)], [(640, 1536), (128, 3328), (200, 776)]
    big = flora.workspace_bytes(flora.matrices(second), r) + flora.workspace_bytes(flora.matrices(first), r)
    ws = torch.empty(4 * big, dtype=torch.uint8, device=DEV)
    x1, x2 = _inputs(first, r, bf16, 1), _inputs(second, r, bf16, 2)
    flora.set_workspace(ws)
    _step_sequence(first, r, bf16, x1)            # the runtime's own lazy set-up happens here
    out2 = _step_sequence(second, r, bf16, x2)    # (and torch's allocator has blocks of these sizes now)
    del out2
    torch.cuda.synchronize()
    third = [(n + 64, m + 128) for n, m in second]
    x3 = _inputs(third, r, bf16, 3)
    outs = [torch.empty(s, device=DEV) for s in third]          # what _step_sequence itself allocates
    del outs
    free_before, _ = torch.cuda.mem_get_info()
    W = [w.clone() for w in x3["W"]]
    free_before, _ = torch.cuda.mem_get_info()
    mats = flora.matrices(third, grads=x3["G"], weights=W, states=x3["M"], row_stats=x3["R"], col_stats=x3["K"],
                          seeds=[3] * 3, seeds_next=[4] * 3)
    flora.fused_step(mats, r, flora.BF16, flora.F32, 0.9, 0.1, True, flora.factored_update(1e-2, 1.0, 0.0, 1e-30, 1.0))
    flora.compress(mats, r, flora.BF16, 0.5, 0.5)
    flora.momentum_transfer(mats, r)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before, (free_before, free_after)
    # the same calls on yet another set, library-allocated: now free memory does go down
    flora.set_workspace(None)
    fourth = [(n + 128, m + 256) for n, m in second]
    x4 = _inputs(fourth, r, bf16, 4)
    W4 = [w.clone() for w in x4["W"]]
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    mats = flora.matrices(fourth, grads=x4["G"], weights=W4, states=x4["M"], row_stats=x4["R"], col_stats=x4["K"],
                          seeds=[3] * 3, seeds_next=[4] * 3)
    flora.fused_step(mats, r, flora.BF16, flora.F32, 0.9, 0.1, True, flora.factored_update(1e-2, 1.0, 0.0, 1e-30, 1.0))
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after < free_before


def test_more_matrices_than_one_launch_takes_with_a_workspace():
    """A call over more matrices than one grouped launch carries seeds for (448) is split into
    chunks; with a workspace every chunk's plan is resident for the call."""
    r, count = 16, 460
    shapes = [(32 + (l % 3) * 16, 64 + (l % 5) * 32) for l in range(count)]
    g = torch.Generator(device="cpu").manual_seed(3)
    G = [torch.randn(*s, generator=g).to(DEV) for s in shapes]
    seeds = [int(flora.derive_seed(8, l, 0)) for l in range(count)]
    need = flora.workspace_bytes(flora.matrices(shapes), r)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = {}
    for mode in ("library", "workspace"):
        flora.set_workspace(ws if mode == "workspace" else None)
        S = [torch.zeros(n, r, device=DEV) for n, _ in shapes]
        flora.compress(flora.matrices(shapes, grads=G, states=S, seeds=seeds), r, flora.F32)
        torch.cuda.synchronize()
        out[mode] = S
    for l in range(count):
        assert torch.equal(out["library"][l], out["workspace"][l])
    for l in (0, 447, 448, 459):
        assert rel_fro(to64(out["workspace"][l]), oracle.compress(to64(G[l]), r, seeds[l])) < tol_for(r)
