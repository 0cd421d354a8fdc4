"""CPU-only checks of the C-ABI boundary: the library loads, exports every
function the headers under include/ declare, and rejects bad arguments on the host
before anything could be launched (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2402_03293_amd import flora, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function any header under include/ declares."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        src = open(os.path.join(inc, fn)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names.update(re.findall(r"\b(flora_[a-z_0-9]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 12
    L = flora.lib()
    for name in names:
        assert hasattr(L, name), name
    assert sorted(flora.EXPORTS) == names


def test_struct_layout_matches_header():
    assert ctypes.sizeof(flora.Matrix) == 5 * 8 + 2 * 8 + 2 * 8 + 2 * 8
    assert ctypes.sizeof(flora.Update) == 10 * 4
    assert flora.Matrix.second_moment.offset == 72 and flora.Matrix.weight_sumsq.offset == 80
    assert flora.Update.scale_parameter.offset == 28 and flora.Update.eps2.offset == 32
    assert flora.Update.step_weight_mib.offset == 36


def test_status_strings_and_version():
    L = flora.lib()
    assert L.flora_status_string(0) == b"ok"
    assert b"invalid" in L.flora_status_string(-1)
    assert b"unsupported" in L.flora_status_string(-2)
    assert flora.version() >= 100


def _mats(n=16, m=16, grad=0x1000, weight=0x2000, state=0x3000, rs=None, cs=None):
    # fake, aligned, non-null device addresses: validation never dereferences them
    return flora.matrices([(n, m)], grads=[grad], weights=[weight], states=[state],
                          row_stats=[rs] if rs else None, col_stats=[cs] if cs else None, seeds=[1])


def test_compress_validation():
    L = flora.lib()
    ok = _mats()
    assert L.flora_compress(None, 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(ok, -1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(ok, 1, 0, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(ok, 1, 12, flora.F32, 1.0, 1.0, None) == flora.ERR_UNSUPPORTED
    assert L.flora_compress(ok, 1, 512, flora.BF16, 1.0, 1.0, None) == flora.ERR_UNSUPPORTED
    assert L.flora_compress(ok, 1, 16, 7, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress_mapped(ok, 1, 16, flora.F32, 2, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress_mapped(ok, 1, 16, flora.F32, -1, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress_mapped(None, 1, 16, flora.F32, flora.INPUT_SQUARE, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress_mapped(ok, 1, 12, flora.F32, flora.INPUT_SQUARE, 1.0, 1.0, None) == flora.ERR_UNSUPPORTED
    assert L.flora_compress(_mats(n=0), 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(_mats(m=-3), 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(_mats(grad=0x1004), 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(_mats(state=0x3008), 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(_mats(grad=0x3000), 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    nog = flora.matrices([(16, 16)], states=[0x3000], seeds=[1])
    assert L.flora_compress(nog, 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
    assert L.flora_compress(ok, 0, 16, flora.F32, 1.0, 1.0, None) == flora.OK      # empty set


def test_decompress_and_transfer_validation():
    L = flora.lib()
    ok = _mats()
    out = (ctypes.c_void_p * 1)(0x4000)
    assert L.flora_decompress(ok, 1, 16, 1.0, None, flora.F32, None) == flora.ERR_INVALID
    assert L.flora_decompress(ok, 1, 16, 1.0, (ctypes.c_void_p * 1)(None), flora.F32, None) == flora.ERR_INVALID
    assert L.flora_decompress(ok, 1, 16, 1.0, (ctypes.c_void_p * 1)(0x4002), flora.F32, None) == flora.ERR_INVALID
    assert L.flora_decompress(ok, 1, 16, 1.0, out, 9, None) == flora.ERR_INVALID
    assert L.flora_decompress(ok, 1, 20, 1.0, out, flora.F32, None) == flora.ERR_UNSUPPORTED
    assert L.flora_decompress(ok, 0, 16, 1.0, None, flora.F32, None) == flora.OK
    assert L.flora_momentum_transfer(None, 2, 16, None) == flora.ERR_INVALID
    assert L.flora_momentum_transfer(ok, 1, 3, None) == flora.ERR_UNSUPPORTED
    nos = flora.matrices([(16, 16)], seeds=[1])
    assert L.flora_momentum_transfer(nos, 1, 16, None) == flora.ERR_INVALID


def test_update_validation():
    L = flora.lib()
    ok = _mats()
    sgd = flora.sgd_update(0.1)
    assert L.flora_apply_update(ok, 1, 16, flora.F32, None, None) == flora.ERR_INVALID
    assert L.flora_apply_update(ok, 1, 16, 2, ctypes.byref(sgd), None) == flora.ERR_INVALID       # no such dtype
    assert L.flora_apply_update(ok, 1, 16, 5, ctypes.byref(sgd), None) == flora.ERR_INVALID
    bad_rule = flora.Update(9, 0.1, 1.0, 0, 0, 0, 0, 0, 0)
    assert L.flora_apply_update(ok, 1, 16, flora.F32, ctypes.byref(bad_rule), None) == flora.ERR_INVALID
    for bad in (-1.0, float("inf"), float("nan")):
        assert L.flora_apply_update(ok, 1, 16, flora.F32, ctypes.byref(flora.sgd_update(0.1, step_weight_mib=bad)),
                                    None) == flora.ERR_INVALID
    fac = flora.factored_update(0.1, 1.0, 0.0, 1e-30, 1.0)
    assert L.flora_apply_update(ok, 1, 16, flora.F32, ctypes.byref(fac), None) == flora.ERR_INVALID  # no R, K
    neg = flora.factored_update(0.1, 1.0, 1.5, 1e-30, 1.0)
    assert L.flora_apply_update(_mats(rs=0x5000, cs=0x6000), 1, 16, flora.F32, ctypes.byref(neg), None) \
        == flora.ERR_INVALID
    now = flora.matrices([(16, 16)], states=[0x3000], seeds=[1])
    assert L.flora_apply_update(now, 1, 16, flora.F32, ctypes.byref(sgd), None) == flora.ERR_INVALID
    assert L.flora_fused_step(ok, 1, 64, flora.F32, 3, 0.9, 0.1, 0, ctypes.byref(sgd), None) == flora.ERR_INVALID
    assert L.flora_fused_step(ok, 0, 64, flora.BF16, flora.F32, 0.9, 0.1, 0, ctypes.byref(sgd), None) == flora.OK


def test_debug_generate_validation():
    L = flora.lib()
    assert L.flora_debug_generate(1, -1, 16, None, None, None) == flora.ERR_INVALID
    assert L.flora_debug_generate(1, 8, 6, 0x1000, None, None) == flora.ERR_INVALID
    assert L.flora_debug_generate(1, 8, 2048, 0x1000, None, None) == flora.ERR_INVALID
    assert L.flora_debug_generate(1, 8, 16, 0x1004, None, None) == flora.ERR_INVALID
    assert L.flora_debug_generate(1, 0, 16, 0x1000, None, None) == flora.OK
    assert L.flora_debug_generate(1, 8, 16, None, None, None) == flora.OK


def test_workspace_query_and_seed_helper_are_host_only():
    wl = workloads.workload(2)
    mats = flora.matrices(wl.shapes)
    b = flora.workspace_bytes(mats, wl.r)
    assert 0 < b < 64 << 20
    assert flora.workspace_bytes(mats, 0) == 0
    s = {flora.derive_seed(7, l, e) for l in range(30) for e in range(30)}
    assert len(s) == 900


def test_workload_tallies_match_the_configurations():
    want = {1: (1, 65536), 2: (96, 44040192), 3: (48, 84934656), 4: (384, 2818572288), 5: (192, 1474560000)}
    for i, (cnt, el) in want.items():
        wl = workloads.workload(i)
        assert (len(wl.shapes), wl.elements) == (cnt, el)
    assert workloads.workload(4).state_elements * 4 == 1384120320


def test_adafactor_rules_validation_and_schedule_helper():
    import ctypes as C
    L = flora.lib()
    base = dict(grads=[0x1000], weights=[0x2000], states=[0x3000], seeds=[1])
    no_v = flora.matrices([(16, 16)], **base)
    with_v = flora.matrices([(16, 16)], second_moments=[0x5000], **base)
    unf = flora.unfactored_update(0.1, 1.0, 0.0, 1e-30, 1.0)
    assert L.flora_apply_update(no_v, 1, 16, flora.F32, C.byref(unf), None) == flora.ERR_INVALID
    scaled = flora.unfactored_update(0.1, 1.0, 0.0, 1e-30, 1.0, scale_parameter=True)
    assert L.flora_apply_update(with_v, 1, 16, flora.F32, C.byref(scaled), None) == flora.ERR_INVALID
    bad_b = flora.unfactored_update(0.1, 1.0, -0.1, 1e-30, 1.0)
    assert L.flora_apply_update(with_v, 1, 16, flora.F32, C.byref(bad_b), None) == flora.ERR_INVALID
    alias = flora.matrices([(16, 16)], second_moments=[0x2000], **base)
    assert L.flora_apply_update(alias, 1, 16, flora.F32, C.byref(unf), None) == flora.ERR_INVALID
    odd = flora.matrices([(16, 16)], second_moments=[0x5004], **base)
    assert L.flora_apply_update(odd, 1, 16, flora.F32, C.byref(unf), None) == flora.ERR_INVALID
    assert L.flora_weight_sumsq(no_v, 1, flora.F32, None) == flora.ERR_INVALID
    assert L.flora_weight_sumsq(None, 1, flora.F32, None) == flora.ERR_INVALID
    assert L.flora_weight_sumsq(no_v, 0, flora.F32, None) == flora.OK
    assert L.flora_weight_sumsq(no_v, 0, 5, None) == flora.ERR_INVALID
    # published schedules: rho_t = min(1e-2, 1/sqrt(t)), beta2_t = 1 - t^-0.8
    assert flora.adafactor_schedule(1) == (pytest.approx(1e-2, rel=1e-6), 0.0)
    assert flora.adafactor_schedule(32)[1] == pytest.approx(0.9375, rel=1e-6)
    assert flora.adafactor_schedule(40000)[0] == pytest.approx(5e-3, rel=1e-6)
    L.flora_adafactor_schedule(5, None, None)          # NULL outputs are allowed


# ---- caller-owned workspace: sizes and validation (host only) --------------------------------
def _round256(x):
    return (x + 255) // 256 * 256


@pytest.mark.parametrize("index,r", [(2, 16), (3, 64), (5, 256), (1, 8)])
def test_workspace_bytes_is_the_sum_of_the_fused_steps_plans(index, r):
    wl = workloads.workload(index)
    shapes = wl.shapes
    mats = flora.matrices(shapes)
    total = flora.workspace_bytes(mats, r)
    comp = max(flora.debug_plan_bytes(0, shapes, r, flora.BF16), flora.debug_plan_bytes(0, shapes, r, flora.F32))
    parts = comp + flora.debug_plan_bytes(3, shapes, r) + flora.debug_plan_bytes(2, shapes, r)
    assert total == max(parts, flora.debug_plan_bytes(4, shapes, r))
    assert total % 256 == 0 and total > 0
    # a plan = its work tables (48 bytes per workgroup) + its work area + 8 descriptor images
    items, info = flora.debug_work_items(1, shapes, r)
    image = _round256(184 * len(shapes))
    assert flora.debug_plan_bytes(1, shapes, r) == _round256(48 * len(items)) + 8 * image
    gdt = flora.F32 if wl.grad_dtype == "f32" else flora.BF16
    items, info = flora.debug_work_items(0, shapes, r, gdt)
    work = _round256(4 * int(info[3])) + 4 * int(info[4])
    assert flora.debug_plan_bytes(0, shapes, r, gdt) == _round256(48 * len(items)) + _round256(work) + 8 * image
    # the transfer's work area: T per matrix, and at ranks >= 64 one partial per chunk of 1024 columns
    t_items, _ = flora.debug_work_items(3, shapes, r)
    a_items, _ = flora.debug_work_items(2, shapes, r)
    twork = sum(_round256(4 * r * r) + (_round256(4 * r * r * ((m + 1023) // 1024)) if r >= 64 else 0) for _, m in shapes)
    assert flora.debug_plan_bytes(2, shapes, r) == (_round256(48 * len(t_items)) + _round256(48 * len(a_items))
                                                    + twork + 8 * image)


def test_workspace_bytes_rejects_bad_sets():
    assert flora.workspace_bytes(flora.matrices([(0, 4)]), 16) == 0
    assert flora.workspace_bytes(flora.matrices([(4, 4)]), 12) == 0
    assert flora.lib().flora_workspace_bytes(None, 1, 16) == 0


def test_set_workspace_validation_and_too_small_is_refused_before_any_device_work():
    L = flora.lib()
    try:
        assert L.flora_set_workspace(0x10001, 4096) == flora.ERR_INVALID         # not 256-byte aligned
        assert L.flora_set_workspace(None, 4096) == flora.ERR_INVALID
        assert L.flora_set_workspace(0x10000, 0) == flora.ERR_INVALID
        # a (fake) workspace of one unit: every call needs more, and says so on the host, before
        # the device is touched (the addresses here are never dereferenced)
        assert L.flora_set_workspace(0x10000, 256) == flora.OK
        ok = _mats(n=64, m=64, rs=0x4000, cs=0x5000)
        upd = flora.sgd_update(1e-3)
        assert L.flora_compress(ok, 1, 16, flora.F32, 1.0, 1.0, None) == flora.ERR_INVALID
        assert L.flora_apply_update(ok, 1, 16, flora.F32, ctypes.byref(upd), None) == flora.ERR_INVALID
        assert L.flora_momentum_transfer(ok, 1, 16, None) == flora.ERR_INVALID
        assert L.flora_fused_step(ok, 1, 16, flora.F32, flora.F32, 0.9, 0.1, 1, ctypes.byref(upd), None) == flora.ERR_INVALID
        # one unit short of what the fused step needs is refused as well
        need = flora.workspace_bytes(ok, 16)
        fac = flora.factored_update(1e-3, 1.0, 0.0, 1e-30, 1.0)
        assert L.flora_set_workspace(0x10000, need - 256) == flora.OK
        assert L.flora_fused_step(ok, 1, 16, flora.F32, flora.F32, 0.9, 0.1, 1, ctypes.byref(fac), None) == flora.ERR_INVALID
    finally:
        assert L.flora_set_workspace(None, 0) == flora.OK


def test_static_transfer_rejects_what_its_buffer_cannot_hold():
    L = flora.lib()
    assert b"fixed scratch" in L.flora_status_string(flora.ERR_TOO_LARGE)
    # 20 matrices of 1600 x 6400 at r = 256 need 20 * 8 * 256 KiB = 40 MiB of T and partials
    big = flora.matrices([(1600, 6400)] * 20, states=[0x3000] * 20, seeds=[1] * 20, seeds_next=[2] * 20)
    assert L.flora_momentum_transfer_static(big, 20, 256, None) == flora.ERR_TOO_LARGE
    many = flora.matrices([(8, 8)] * 449, states=[0x3000] * 449)
    assert L.flora_momentum_transfer_static(many, 449, 8, None) == flora.ERR_TOO_LARGE
    assert L.flora_momentum_transfer_static(None, 1, 8, None) == flora.ERR_INVALID
    assert L.flora_momentum_transfer_static(many, 1, 12, None) == flora.ERR_UNSUPPORTED
    assert L.flora_momentum_transfer_static(many, 0, 8, None) == flora.OK
