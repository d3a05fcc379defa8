"""CPU tests of the library's host side: exported symbols, the planner's decomposition
(against Table 3 and the paper's printed 5x5 examples), layout bookkeeping and error
codes.  No compute call is made, so no GPU is needed."""
import ctypes
import os
import re

import numpy as np
import pytest

import dwm_workloads as wl
import paper_2002_00552_amd as dwm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dwm.h")).read()
    declared = sorted(set(re.findall(r"DWM_API[^;(]*?\b(dwm_\w+)\s*\(", header)))
    assert len(declared) >= 14
    raw = ctypes.CDLL(dwm.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert declared == dwm.EXPORTS  # the binding carries the same names


def test_probe_library_exports_its_entry_points():
    """The peak probes beside bench.py (their own library): every PROBE_API function is exported, and the
    operand-delivery probe refuses arguments that would take its addresses outside its buffers."""
    import bench_probes
    if not os.path.exists(bench_probes.PROBE_LIB):
        bench_probes.build()
    src = open(os.path.join(ROOT, "bench_probes.hip")).read()
    declared = sorted(set(re.findall(r"PROBE_API\s+int\s+(dwm_probe_\w+)\s*\(", src)))
    assert declared == ["dwm_probe_copy", "dwm_probe_fill", "dwm_probe_mfma", "dwm_probe_mix", "dwm_probe_read"]
    L = bench_probes.lib()
    for name in declared:
        assert hasattr(L, name), name
    # refused on the host, before anything is launched: too many workgroups, a mask that is not 2^n - 1, a stream
    # stride whose 128 streams would not fit
    assert L.dwm_probe_mix(None, None, 0, 1, 257, 0, (1 << 20) - 1, None) == 1
    assert L.dwm_probe_mix(None, None, 0, 1, 196, 0, (1 << 20), None) == 1
    assert L.dwm_probe_mix(None, None, 0, 1, 196, (1 << 24) + 1, (1 << 20) - 1, None) == 1
    assert L.dwm_probe_mix(None, None, 9, 0, 196, 0, (1 << 20) - 1, None) == 1


def _plan(*a):
    p = dwm.dwm_plan_create(*a)
    return p, dwm.dwm_plan_info(p)


def test_table3_counts_from_the_planner(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "table3_mults.txt"))
            if l.strip() and not l.startswith("#")]
    for k, s, direct_p, dwm_p, speed_p in rows:
        k, s = int(k), int(s)
        # 14x14 output: H chosen so that OH = 14 with same-style padding
        H = 14 * s
        p, info = _plan(1, 1, H, H, 1, k, k, s, k // 2)
        assert info.OH >= 14 - 1
        m = info.mults_per_tile
        assert abs(49 * m - float(dwm_p)) <= 0.5 * 10 ** max(len(str(49 * m)) - 3, 0), (k, s, m)
        assert abs(196 * k * k / (49 * m) - float(speed_p)) <= 0.005 + 1e-9
        dwm.dwm_plan_destroy(p)


@pytest.mark.parametrize("stride", [1, 2])
def test_5x5_splits_as_the_paper_says(stride):
    p, info = _plan(1, 1, 16, 16, 1, 5, 5, stride, 2)
    sizes = sorted((dwm.dwm_plan_part(p, i).len_h, dwm.dwm_plan_part(p, i).len_w) for i in range(info.n_parts))
    assert sizes == [(2, 2), (2, 3), (3, 2), (3, 3)]
    dwm.dwm_plan_destroy(p)


@pytest.mark.parametrize("R,S,s", [(r, q, s) for r in (1, 2, 3, 5, 7, 8, 11, 12) for q in (1, 3, 4, 7, 11)
                                   for s in (1, 2, 3, 4, 6)])
def test_taps_partition_and_layout(R, S, s):
    C, K = 5, 7
    p, info = _plan(2, C, 40, 41, K, R, S, s, 3)
    cover = np.zeros((R, S), int)
    classes = [dwm.dwm_plan_class(p, i) for i in range(info.n_classes)]
    slots = {}
    mults = 0
    for i in range(info.n_parts):
        pt = dwm.dwm_plan_part(p, i)
        q = classes[pt.cls]
        assert (q.len_h, q.len_w) == (pt.len_h, pt.len_w)
        assert 0 <= pt.slot < q.n_parts and (pt.cls, pt.slot) not in slots
        slots[(pt.cls, pt.slot)] = i
        assert pt.phase_h < s and pt.phase_w < s
        mults += (pt.len_h + 1) * (pt.len_w + 1)
        for a in range(pt.len_h):
            for b in range(pt.len_w):
                cover[s * (pt.off_h + a) + pt.phase_h, s * (pt.off_w + b) + pt.phase_w] += 1
    assert np.all(cover == 1)
    assert mults == info.mults_per_tile
    assert info.n_planes == sum((q.len_h + 1) * (q.len_w + 1) for q in classes)
    # classes tile the two buffers without overlap
    u_end = v_end = 0
    for q in classes:
        assert q.L == q.n_parts * C and q.Lpad >= q.L and q.Lpad % 16 == 0
        assert q.u_offset == u_end and q.v_offset == v_end
        planes = (q.len_h + 1) * (q.len_w + 1)
        u_end += planes * info.Kpad * q.Lpad
        v_end += planes * q.Lpad * 64  # offsets inside one block of 64 tiles
    # V comes first in the workspace; partial tiles and counters of the contraction follow
    assert info.Vblock == v_end and info.Tpad % 64 == 0
    assert dwm.dwm_plan_workspace_bytes(p) >= 4 * info.Vblock * (info.Tpad // 64)
    # the single-kernel path's filter copy follows (few input channels: it applies here)
    nfc, nrows, nslices = dwm.dwm_plan_fused_info(p)
    if nfc == 0:
        assert dwm.dwm_plan_filter_bytes(p) == 4 * u_end
    else:
        assert nslices == (K + 31) // 32
        uf_end, row_end, seen = u_end, 0, set()
        for i in range(nfc):
            fq = dwm.dwm_plan_fused_class(p, i)
            assert fq.uf_offset >= uf_end and fq.uf_offset % 2 == 0 and fq.rows % 4 == 0
            assert fq.first_row == row_end and (fq.n_freq_h, fq.n_freq_w) == (4 if fq.wide_h else 2, 4 if fq.wide_w else 2)
            for r in range(fq.first_row, fq.first_row + fq.rows):
                row = dwm.dwm_plan_fused_row(p, r)
                pt = dwm.dwm_plan_part(p, row.part)
                assert (pt.len_h >= 2) == bool(fq.wide_h) and (pt.len_w >= 2) == bool(fq.wide_w)
                assert 0 <= row.channel < C
                if row.real:
                    assert (row.part, row.channel) not in seen
                    seen.add((row.part, row.channel))
            row_end += fq.rows
            uf_end = fq.uf_offset + nslices * fq.n_freq_h * fq.n_freq_w * fq.rows * 32
        assert row_end == nrows and len(seen) == info.n_parts * C  # every (part, channel) exactly once
        assert dwm.dwm_plan_filter_bytes(p) == 4 * uf_end
        # with this path, one-tap pieces only come from phases that hold a single tap
        for i in range(info.n_parts):
            pt = dwm.dwm_plan_part(p, i)
            if pt.len_h == 1:
                assert pt.off_h == 0 and s * 1 + pt.phase_h >= R
            if pt.len_w == 1:
                assert pt.off_w == 0 and s * 1 + pt.phase_w >= S
    assert info.Kpad >= K and info.Tpad >= info.T == 2 * info.TH * info.TW
    dwm.dwm_plan_destroy(p)


def test_benchmark_configs_plan_as_expected():
    want = {0: (4, 49), 1: (4, 25), 2: (9, 100), 3: (9, 100), 4: (16, 225)}
    for i, L in enumerate(wl.CONFIGS):
        p, info = _plan(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
        assert (info.n_parts, info.mults_per_tile) == want[i]
        assert info.direct_flops == wl.direct_flops(L)
        assert (info.OH, info.OW) == wl.out_hw(L)
        dwm.dwm_plan_destroy(p)


def test_error_codes():
    h = ctypes.c_void_p()
    L = dwm.lib()
    ok = (1, 1, 8, 8, 1, 3, 3, 1, 1)
    assert L.dwm_plan_create(None, *ok) == dwm.DWM_ERR_INVALID_ARG
    for pos in range(7):
        bad = list(ok)
        bad[pos] = 0
        assert L.dwm_plan_create(ctypes.byref(h), *bad) == dwm.DWM_ERR_INVALID_ARG, pos
    assert L.dwm_plan_create(ctypes.byref(h), 1, 1, 8, 8, 1, 3, 3, 0, 1) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_plan_create(ctypes.byref(h), 1, 1, 8, 8, 1, 3, 3, 1, -1) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_plan_create(ctypes.byref(h), 1, 1, 2, 2, 1, 3, 3, 1, 0) == dwm.DWM_ERR_INVALID_ARG  # empty output
    assert L.dwm_plan_create(ctypes.byref(h), 1, 1, 80, 80, 1, 49, 3, 1, 0) == dwm.DWM_ERR_UNSUPPORTED  # 17 pieces
    assert L.dwm_plan_create(ctypes.byref(h), 1, 1, 80, 80, 1, 48, 3, 1, 0) == dwm.DWM_OK
    plan = h
    # no workspace yet: every stage that needs it refuses before touching the GPU
    one = ctypes.c_void_p(256)
    assert L.dwm_conv_forward(plan, one, one, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_input_transform(plan, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_contract_output(plan, one, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_conv_forward(plan, None, one, one, None) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_filter_transform(plan, None, one, None) == dwm.DWM_ERR_INVALID_ARG
    need = dwm.dwm_plan_workspace_bytes(plan)
    assert L.dwm_plan_set_workspace(plan, ctypes.c_void_p(4096), need - 1) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_plan_set_workspace(plan, ctypes.c_void_p(4096 + 4), need) == dwm.DWM_ERR_WORKSPACE  # misaligned
    assert L.dwm_plan_set_workspace(plan, None, need) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_plan_set_variant(plan, b"nonsense", 0) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_plan_part(plan, 10 ** 6, ctypes.byref(dwm.dwm_part_t())) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_plan_destroy(plan) == dwm.DWM_OK
    assert L.dwm_plan_destroy(None) == dwm.DWM_ERR_INVALID_ARG
    with pytest.raises(dwm.DwmError):
        dwm.dwm_plan_create(0, 1, 1, 1, 1, 1, 1, 1, 0)
    assert "workspace" in dwm.dwm_status_string(dwm.DWM_ERR_WORKSPACE)


# ---------------------------------------------------------------------------------------
# half-precision plan (host side only)
# ---------------------------------------------------------------------------------------
def test_half_plan_is_cut_as_printed():
    """The half-precision plan cuts the kernel 3,3,...,remainder (eq. 8) on every layer, also
    where the single-precision planner prefers 2+2 tails: the parts are the oracle's parts."""
    import oracle
    for L in wl.CONFIGS + [wl.Layer("k4", 1, 8, 20, 20, 8, 4, 4, 1, 1, "uniform")]:
        p = dwm.dwm_f16_plan_create(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
        info = dwm.dwm_f16_plan_info(p)
        parts = oracle.split_2d(L.R, L.S, L.stride)
        assert info.n_parts == len(parts)
        assert info.mults_per_tile == oracle.mults_per_tile(L.R, L.S, L.stride)
        # the 16-bit single kernel where the layer has few input channels, else the staged path
        assert info.forward_path == (1 if L.C <= 16 else 0)
        dwm.dwm_f16_set_variant(p, "forward", 0)
        assert dwm.dwm_f16_plan_info(p).forward_path == 0
        # U16 holds every plane's Kpad x Lpad block, two bytes per element (and the single kernel's copy
        # behind it where that path applies)
        assert dwm.dwm_f16_filter_bytes(p) % 256 == 0
        assert dwm.dwm_f16_filter_bytes(p) >= 2 * info.mults_per_tile * L.C * L.K
        # workspace: V16 (all planes' rows for Tpad tiles) and then some
        assert dwm.dwm_f16_workspace_bytes(p) >= 2 * info.mults_per_tile * L.C * info.T
        dwm.dwm_f16_plan_destroy(p)


def test_half_plan_error_codes():
    L = dwm.lib()
    h = ctypes.c_void_p()
    assert L.dwm_f16_plan_create(None, 1, 1, 8, 8, 1, 3, 3, 1, 1) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_plan_create(ctypes.byref(h), 1, 1, 8, 8, 1, 3, 3, 0, 1) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_plan_create(ctypes.byref(h), 1, 1, 2, 2, 1, 3, 3, 1, 0) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_plan_create(ctypes.byref(h), 1, 1, 80, 80, 1, 49, 3, 1, 0) == dwm.DWM_ERR_UNSUPPORTED
    assert L.dwm_f16_plan_create(ctypes.byref(h), 2, 64, 16, 16, 128, 3, 3, 1, 1) == dwm.DWM_OK
    plan = h
    one = ctypes.c_void_p(256)
    assert L.dwm_f16_conv_forward(plan, one, one, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_f16_conv_forward_f32out(plan, one, one, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_f16_input_transform(plan, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_f16_contract_output(plan, one, one, None) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_f16_conv_forward(plan, None, one, one, None) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_filter_transform(plan, one, None, None) == dwm.DWM_ERR_INVALID_ARG
    need = dwm.dwm_f16_workspace_bytes(plan)
    assert L.dwm_f16_set_workspace(plan, ctypes.c_void_p(4096), need - 1) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_f16_set_workspace(plan, ctypes.c_void_p(4096 + 8), need) == dwm.DWM_ERR_WORKSPACE
    assert L.dwm_f16_set_workspace(plan, None, need) == dwm.DWM_ERR_WORKSPACE
    # variants: single-precision ids are refused, half-precision ids that fit are accepted, and
    # one that needs more partial-output space than the workspace handed over holds is refused
    assert L.dwm_f16_set_variant(plan, b"contract", 12) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_set_variant(plan, b"contract", 48) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_set_variant(plan, b"nonsense", 30) == dwm.DWM_ERR_INVALID_ARG
    for v in range(30, 48):
        assert L.dwm_f16_set_variant(plan, b"contract", v) == dwm.DWM_OK, v
    assert L.dwm_f16_set_variant(plan, b"contract", -1) == dwm.DWM_OK
    assert L.dwm_f16_set_variant(plan, b"input", 0) == dwm.DWM_OK
    assert L.dwm_f16_set_variant(plan, b"input", 1) == dwm.DWM_OK
    assert L.dwm_f16_set_variant(plan, b"input", 2) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_plan_set_variant(ctypes.c_void_p(0), b"contract", 30) == dwm.DWM_ERR_INVALID_ARG
    assert L.dwm_f16_plan_destroy(plan) == dwm.DWM_OK
    assert L.dwm_f16_plan_destroy(None) == dwm.DWM_ERR_INVALID_ARG
    # a half-precision contraction id is not a single-precision variant
    p32 = dwm.dwm_plan_create(2, 64, 16, 16, 128, 3, 3, 1, 1)
    assert L.dwm_plan_set_variant(p32, b"contract", 32) == dwm.DWM_ERR_INVALID_ARG
    dwm.dwm_plan_destroy(p32)


def test_workspace_holds_the_partial_outputs_of_tiles_cut_into_ranges():
    """With at most one tile per CU, and long tiles, the contraction cuts every tile into 2..8
    ranges of its own (about two workgroups per CU, no range under 16 chunks): the workspace then
    holds that many 64x64x(2x2) partial outputs per tile after V.  With short tiles (few chunks)
    or more tiles than CUs it does not."""
    def extra(shape):
        p = dwm.dwm_plan_create(*shape)
        info = dwm.dwm_plan_info(p)
        e = dwm.dwm_plan_workspace_bytes(p) - 4 * info.Vblock * (info.Tpad // 64)
        tiles = ((info.K + 63) // 64) * ((info.T + 63) // 64)
        dwm.dwm_plan_destroy(p)
        return e, tiles
    slot = 64 * 64 * 4 * 4
    e, tiles = extra((3, 16, 56, 56, 256, 5, 5, 1, 2))   # 49 chunks: three ranges of 17, 17, 15
    assert tiles == 148 and tiles * 3 * slot <= e < tiles * 4 * slot
    e, tiles = extra((1, 16, 56, 56, 256, 5, 5, 1, 2))   # 52 tiles: 512 / 52 = 9 -> 8, but 49 / 16 = 3 ranges
    assert tiles == 52 and tiles * 3 * slot <= e < tiles * 4 * slot
    e, tiles = extra((3, 16, 56, 56, 256, 3, 3, 1, 1))   # 16 chunks per tile: whole tiles
    assert tiles == 148 and e < slot
    e, tiles = extra((8, 16, 56, 56, 256, 5, 5, 1, 2))   # 392 tiles: one round of whole tiles + ranges
    assert tiles == 392 and e < tiles * 2 * slot
