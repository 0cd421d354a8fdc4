"""Host logic without a GPU: the tables of workgroups behind the grouped launches.

Whatever the shapes, every element of every matrix must belong to exactly one workgroup of a
launch (per rank slice for compression), the workgroups that share the columns of a row block
must agree on where their partial products and their arrival counter live, and no two groups
may share either.  The tables come from the library's own builders through a host-only hook.
"""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from paper_2402_03293_amd import flora, workloads

COLS = dict(mat=0, row0=1, rows=2, col0=3, slice=4, rblock=5, col1=6, part=7, nparts=8, cidx=9, poff=10)
RANKS = [8, 16, 32, 64, 128, 256]

shape_lists = st.lists(st.tuples(st.integers(1, 5000), st.integers(1, 9000)), min_size=1, max_size=5)
aligned_shape_lists = st.lists(st.tuples(st.integers(1, 5000), st.integers(1, 1100).map(lambda x: 8 * x)),
                               min_size=1, max_size=5)


def check_compress(shapes, r, gdt):
    items, info = flora.debug_work_items(0, shapes, r, gdt)
    mt, _, kc, ws_floats, ws_counters = (int(x) for x in info)
    c = COLS
    if r <= 32:
        rows_per_wg, slice_w, nslices, rp = 64 * mt, None, 1, max(16, r)
    else:
        wide = mt >= 8
        rows_per_wg = 512 if mt == 8 else 256 if mt == 16 else 128 if mt == 32 else 128 * mt
        slice_w = (64 if r == 64 else 128) if wide else 64
        nslices, rp = r // slice_w, slice_w
    groups = {}
    for i, it in enumerate(items):
        groups.setdefault((it[c["mat"]], it[c["rblock"]], it[c["slice"]] if r > 32 else 0), []).append(it)
    # rows: per (matrix, slice) the row blocks tile [0, n)
    for l, (n, m) in enumerate(shapes):
        for s in range(nslices):
            blocks = sorted({(g[0][c["row0"]], g[0][c["rows"]]) for k, g in groups.items() if k[0] == l and k[2] == s})
            assert blocks, (l, s)
            pos = 0
            for row0, rows in blocks:
                assert row0 == pos and 1 <= rows <= rows_per_wg
                pos += rows
            assert pos == n
    seen_counters, spans = set(), []
    for key, g in groups.items():
        n, m = shapes[key[0]]
        g = sorted(g, key=lambda it: it[c["part"]])
        nparts = g[0][c["nparts"]]
        assert [it[c["part"]] for it in g] == list(range(nparts)) and nparts >= 1
        pos = 0
        for it in g:
            assert it[c["nparts"]] == nparts and it[c["row0"]] == g[0][c["row0"]] and it[c["rows"]] == g[0][c["rows"]]
            assert it[c["col0"]] == pos and it[c["col0"]] % 64 == 0 and it[c["col1"]] > it[c["col0"]]
            pos = it[c["col1"]]
        assert pos == m
        if nparts > 1:
            assert len({it[c["cidx"]] for it in g}) == 1 and len({it[c["poff"]] for it in g}) == 1
            cidx, poff = g[0][c["cidx"]], g[0][c["poff"]]
            assert 0 <= cidx < ws_counters and cidx not in seen_counters
            seen_counters.add(cidx)
            spans.append((poff, poff + nparts * rows_per_wg * rp))
    spans.sort()
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0
    if spans:
        assert spans[0][0] >= 0 and spans[-1][1] <= ws_floats
    assert len(seen_counters) == ws_counters
    return items, info


def check_decompress(shapes, r):
    items, info = flora.debug_work_items(1, shapes, r)
    vec = int(info[1])
    cols = 256 if vec else 128
    c = COLS
    if vec:
        assert r >= 64 and all(m % 4 == 0 for _, m in shapes)
    per_mat = {}
    for it in items:
        per_mat.setdefault(it[c["mat"]], []).append(it)
    assert sorted(per_mat) == list(range(len(shapes)))
    for l, (n, m) in enumerate(shapes):
        its = per_mat[l]
        nchunks = (m + cols - 1) // cols
        blocks = sorted({(it[c["rblock"]], it[c["row0"]], it[c["rows"]]) for it in its})
        pos = 0
        for rb, (rblock, row0, rows) in enumerate(blocks):
            assert rblock == rb and row0 == pos and rows >= 1
            if rb + 1 < len(blocks):
                assert rows % 32 == 0
            pos += rows
        assert pos == n
        assert len(its) == len(blocks) * nchunks
        assert sorted(it[c["part"]] for it in its) == list(range(len(its)))       # slots of per-workgroup sums
        for it in its:
            cc = it[c["slice"]]
            assert 0 <= cc < nchunks and it[c["col0"]] == cc * cols
            assert it[c["part"]] == it[c["rblock"]] * nchunks + cc
    return items, info


@settings(max_examples=60, deadline=None)
@given(shape_lists, st.sampled_from([8, 16, 32]), st.sampled_from([flora.F32, flora.BF16]))
def test_fp32_compress_tables_cover_every_element_once(shapes, r, gdt):
    check_compress(shapes, r, gdt)


@settings(max_examples=60, deadline=None)
@given(st.one_of(shape_lists, aligned_shape_lists), st.sampled_from([64, 128, 256]))
def test_bf16_compress_tables_cover_every_element_once(shapes, r):
    check_compress(shapes, r, flora.BF16)


@settings(max_examples=60, deadline=None)
@given(st.one_of(shape_lists, aligned_shape_lists), st.sampled_from(RANKS))
def test_decompress_tables_cover_every_element_once(shapes, r):
    check_decompress(shapes, r)


@settings(max_examples=30, deadline=None)
@given(shape_lists, st.sampled_from(RANKS))
def test_transfer_row_blocks(shapes, r):
    items, _ = flora.debug_work_items(2, shapes, r)
    for l, (n, m) in enumerate(shapes):
        its = sorted((it[1], it[2]) for it in items if it[0] == l)
        pos = 0
        for row0, rows in its:
            assert row0 == pos and 1 <= rows <= (64 if r >= 64 else 32)
            pos += rows
        assert pos == n
    # T = A^T A' at ranks 64 and above: every slab of rows of T sees every column exactly once
    titems, _ = flora.debug_work_items(3, shapes, r)
    if r < 64:
        assert len(titems) == 0
        return
    slabs = r // min(r, 128)
    for l, (n, m) in enumerate(shapes):
        for s_ in range(slabs):
            its = sorted((it[7], it[3], it[6]) for it in titems if it[0] == l and it[4] == s_)
            pos = 0
            for c, (part, col0, col1) in enumerate(its):
                assert part == c and col0 == pos and col0 < col1 <= col0 + 1024
                pos = col1
            assert pos == m


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_tables_of_the_five_workloads(index):
    wl = workloads.workload(index)
    gdt = flora.F32 if wl.grad_dtype == "f32" else flora.BF16
    items, info = check_compress(wl.shapes, wl.r, gdt)
    ditems, dinfo = check_decompress(wl.shapes, wl.r)
    if wl.r >= 64:
        assert int(info[0]) >= 8 and int(dinfo[1]) == 1          # wide compress, 16-byte decompress
    # launches of the full-size workloads fill the chip: more workgroups than compute units
    if index >= 2:
        assert len(items) >= 256 and len(ditems) >= 256


def test_row_blocks_of_a_bundle_share_an_xcd():
    # workgroup ids go round-robin over 8 XCDs: the column chunks of one row block of the state
    # (decompress) are placed 8 apart so that they meet in one L2
    shapes = [(2048, 2048)] * 4
    items, _ = flora.debug_work_items(1, shapes, 256)
    where = {}
    for i, it in enumerate(items):
        where.setdefault((it[0], it[5]), set()).add(i % 8)
    assert all(len(v) == 1 for v in where.values())


def test_hook_rejects_bad_arguments():
    L = flora.lib()
    mats = flora.matrices([(4, 4)])
    assert L.flora_debug_work_items(0, mats, 1, 12, 0, None, 0, None) == flora.ERR_UNSUPPORTED
    assert L.flora_debug_work_items(7, mats, 1, 16, 0, None, 0, None) == flora.ERR_INVALID
    assert L.flora_debug_work_items(0, flora.matrices([(0, 4)]), 1, 16, 0, None, 0, None) == flora.ERR_INVALID
    assert L.flora_debug_work_items(0, mats, 1, 16, 0, None, 0, None) == 1
