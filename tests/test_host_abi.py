"""Host-side checks of libdgc that need no GPU: the library loads, exports what the
header declares, validates arguments before touching the device, and its host
arithmetic (k_j, sample plan, warm-up table) agrees with the oracle's."""

import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dgc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dgc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(dgc_lib):
    names = declared_functions()
    assert "dgc_compress" in names and "dgc_decompress_accumulate" in names and "dgc_set_density" in names
    for name in names:
        assert hasattr(dgc_lib, name), name
    assert sorted(B.EXPORTS) == names
    assert dgc_lib.dgc_version() >= 1000


def test_config_default_and_struct_layout(dgc_lib):
    cfg = B.dgc_config_default()
    assert C.sizeof(B.DgcConfig) == 64
    assert abs(cfg.momentum - 0.9) < 1e-7 and cfg.clip_threshold == 0.0 and cfg.num_workers == 1
    assert cfg.density == 0.001 and cfg.sample_ratio == 0.01
    assert (cfg.sample_min, cfg.sample_max, cfg.sample_block) == (4096, 32768, 32)
    assert math.isnan(cfg.scale_override) and cfg.seed == 0 and cfg.refine_alpha == 0.0


def test_create_rejects_bad_arguments(dgc_lib):
    def create(cfg, offsets):
        h = C.c_void_p()
        arr = (C.c_int64 * len(offsets))(*offsets)
        return dgc_lib.dgc_create(C.byref(h), C.byref(cfg), len(offsets) - 1, arr), h

    ok, h = create(B.dgc_config_default(), [0, 10, 30])
    assert ok == B.DGC_OK
    assert dgc_lib.dgc_destroy(h) == B.DGC_OK
    for bad in ([1, 10], [0, 10, 10], [0, 10, 5]):
        assert create(B.dgc_config_default(), bad)[0] == B.DGC_ERR_INVALID_ARG
    assert create(B.dgc_config_default(), [0, 1 << 31])[0] == B.DGC_ERR_CAPACITY
    for field, value in [("density", 0.0), ("density", 1.5), ("density", float("nan")), ("num_workers", 0),
                         ("momentum", -0.1), ("sample_block", 3), ("sample_block", 128),
                         ("sample_min", 8), ("sample_ratio", 0.0), ("refine_alpha", 0.5), ("refine_alpha", -1.0)]:
        cfg = B.dgc_config_default()
        setattr(cfg, field, value)
        assert create(cfg, [0, 100])[0] == B.DGC_ERR_INVALID_ARG, field
    assert dgc_lib.dgc_create(None, C.byref(B.dgc_config_default()), 1, (C.c_int64 * 2)(0, 4)) == B.DGC_ERR_INVALID_ARG
    assert dgc_lib.dgc_status_string(B.DGC_ERR_CAPACITY) == b"capacity exceeded"


def test_compress_and_accumulate_validate_before_touching_the_device(dgc_lib):
    d = B.Dgc(B.dgc_config_default(), [0, 64, 5000])
    lay = (C.c_int64 * 3)(0, 64, 1000)
    f = dgc_lib.dgc_compress
    # null buffers
    assert f(d._h, None, None, None, None, None, lay, None, None, 0, None, 0, None) == B.DGC_ERR_INVALID_ARG
    # misaligned g (fake non-null addresses are never dereferenced: checks come first)
    a = 0x10000
    assert f(d._h, a + 4, a, a, a, a, lay, a, None, 0, a, 1 << 20, None) == B.DGC_ERR_ALIGNMENT
    # bad payload layout
    bad = (C.c_int64 * 3)(0, 64, 10)
    assert f(d._h, a, a, a, a, a, bad, a, None, 0, a, 1 << 20, None) == B.DGC_ERR_INVALID_ARG
    # workspace missing / misaligned / too small
    assert f(d._h, a, a, a, a, a, lay, a, None, 0, None, 1 << 20, None) == B.DGC_ERR_INVALID_ARG
    assert f(d._h, a, a, a, a, a, lay, a, None, 0, a + 8, 1 << 20, None) == B.DGC_ERR_ALIGNMENT
    assert f(d._h, a, a, a, a, a, lay, a, None, 0, a, 16, None) == B.DGC_ERR_CAPACITY
    acc = dgc_lib.dgc_decompress_accumulate
    ptrs = (C.c_void_p * 1)(a)
    cnt = (C.c_int64 * 1)(5)
    assert acc(d._h, None, 10, 1, ptrs, ptrs, cnt, None, None) == B.DGC_ERR_INVALID_ARG
    assert acc(d._h, a, 0, 1, ptrs, ptrs, cnt, None, None) == B.DGC_ERR_INVALID_ARG
    assert acc(d._h, a, 10, 0, ptrs, ptrs, cnt, None, None) == B.DGC_ERR_INVALID_ARG
    assert acc(d._h, a, 10, 65, ptrs, ptrs, cnt, None, None) == B.DGC_ERR_CAPACITY
    neg = (C.c_int64 * 1)(-1)
    assert acc(d._h, a, 10, 1, ptrs, ptrs, neg, None, None) == B.DGC_ERR_INVALID_ARG
    # the region-layout receive calls: payload lists, previous lists, layout and workspace are checked first
    rep = dgc_lib.dgc_decompress_replace_regions
    big = (C.c_void_p * 65)(*([a] * 65))
    assert rep(d._h, None, 1, ptrs, ptrs, ptrs, 0, None, None, lay, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 0, ptrs, ptrs, ptrs, 0, None, None, lay, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 65, big, big, big, 0, None, None, lay, a, 1 << 24, None) == B.DGC_ERR_CAPACITY
    assert rep(d._h, a, 1, ptrs, None, ptrs, 0, None, None, lay, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 1, ptrs, ptrs, ptrs, -1, None, None, lay, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 1, ptrs, ptrs, ptrs, 1, None, None, lay, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 1, ptrs, ptrs, ptrs, 65, big, big, lay, a, 1 << 24, None) == B.DGC_ERR_CAPACITY
    assert rep(d._h, a, 1, ptrs, ptrs, ptrs, 1, ptrs, ptrs, bad, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 1, ptrs, ptrs, ptrs, 1, ptrs, ptrs, lay, None, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert rep(d._h, a, 1, ptrs, ptrs, ptrs, 1, ptrs, ptrs, lay, a, 16, None) == B.DGC_ERR_CAPACITY
    d.close()


@pytest.mark.parametrize("density", [0.001, 0.004, 0.015625, 0.0625, 0.25, 1.0])
def test_plan_matches_oracle_arithmetic(dgc_lib, density):
    for gs in (S.resnet50_set(), S.speech_set(), S.lstm_lm_set(), S.ragged_set(1), S.toy_set()):
        d = B.Dgc(B.make_config(density=density), gs.offsets)
        ocfg = O.OracleConfig(density=density)
        for j, n in enumerate(gs.sizes):
            k, count, rank, draws = d.dgc_query_plan(j)
            p = O.sample_plan(n, ocfg)
            assert (k, count, rank, draws) == (p.k, p.count, p.rank, p.blocks), (gs.name, j, n)
        d.close()


def test_resnet50_k_sum_and_toy_plan(dgc_lib):
    gs = S.resnet50_set()
    d = B.Dgc(B.dgc_config_default(), gs.offsets)
    assert sum(d.dgc_query_plan(j)[0] for j in range(len(gs.sizes))) == 25670
    lay = d.dgc_recommended_payload_layout(0.001)
    assert lay[0] == 0 and len(lay) == 162
    for j, n in enumerate(gs.sizes):
        k = O.topk_count(0.001, n)
        assert lay[j + 1] - lay[j] == min(n, max(8 * k, k + 256))
    d.close()
    t = B.Dgc(B.dgc_config_default(), [0, 1 << 20])
    assert t.dgc_query_plan(0) == (1049, 10496, 11, 328)
    t.close()


def test_exact_select_flag_uses_whole_tensor(dgc_lib):
    d = B.Dgc(B.make_config(flags=B.DGC_FLAG_EXACT_SELECT), [0, 100000])
    assert d.dgc_query_plan(0) == (100, 100000, 100, 0)
    d.close()


def test_density_control_and_warmup(dgc_lib):
    d = B.Dgc(B.dgc_config_default(), [0, 4723200])
    seen = []
    for it in range(8):
        d.dgc_set_iteration_density(it)
        seen.append(d.dgc_query_plan(0)[0])
    expect = [O.topk_count(O.warmup_density(O.WARMUP_DENSITIES, it), 4723200) for it in range(8)]
    assert seen == expect and seen[0] == 1180800 and seen[-1] == 4724
    d.dgc_set_warmup_schedule([0.5, 0.1])
    d.dgc_set_iteration_density(0)
    assert d.dgc_query_plan(0)[0] == 2361600
    d.dgc_set_iteration_density(9)
    assert d.dgc_query_plan(0)[0] == 472320
    # every entry held for an "epoch" of 391 iterations (Section 4.1: one warm-up sparsity per epoch)
    d.dgc_set_warmup_schedule(list(O.WARMUP_DENSITIES))
    d.dgc_set_warmup_stage_length(391)
    for it, stage in [(0, 0), (390, 0), (391, 1), (4 * 391 - 1, 3), (4 * 391, 4), (10 ** 6, 4)]:
        d.dgc_set_iteration_density(it)
        assert d.dgc_query_plan(0)[0] == O.topk_count(O.WARMUP_DENSITIES[stage], 4723200)
        assert O.warmup_density(O.WARMUP_DENSITIES, it, 391) == O.WARMUP_DENSITIES[stage]
    with pytest.raises(B.DgcError):
        d.dgc_set_warmup_stage_length(0)
    with pytest.raises(B.DgcError):
        d.dgc_set_density(0.0)
    with pytest.raises(B.DgcError):
        d.dgc_set_density(1.01)
    with pytest.raises(B.DgcError):
        d.dgc_set_warmup_schedule([0.5, 0.0])
    with pytest.raises(B.DgcError):
        d.dgc_query_plan(1)
    assert d.dgc_workspace_bytes() > 0 and d.dgc_workspace_bytes() % 256 == 0
    # the warm-up workspace: the same, and behind it two staging arrays of n floats
    extra = d.dgc_workspace_bytes_warmup() - d.dgc_workspace_bytes()
    assert 8 * d.n <= extra <= 8 * d.n + 512 and d.dgc_workspace_bytes_warmup() % 256 == 0
    d.close()


def test_wire_format_entry_points_validate_before_touching_the_device(dgc_lib):
    d = B.Dgc(B.dgc_config_default(), [0, 64, 200000])
    assert d.dgc_encode_max_entries(0) == 3 and d.dgc_encode_max_entries(1000) == 1003   # 200000 >> 16 fillers
    lay = (C.c_int64 * 3)(0, 64, 1000)
    a = 0x10000
    n32 = C.c_void_p(a)
    enc = dgc_lib.dgc_encode
    assert enc(d._h, None, a, a, lay, a, a, 10, a, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert enc(d._h, a, a, a, lay, a, a, -1, a, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert enc(d._h, a, a, a, lay, a + 1, a, 10, a, a, 1 << 24, None) == B.DGC_ERR_ALIGNMENT
    bad = (C.c_int64 * 3)(0, 64, 10)
    assert enc(d._h, a, a, a, bad, a, a, 10, a, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert enc(d._h, a, a, a, lay, a, a, 10, a, None, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert enc(d._h, a, a, a, lay, a, a, 10, a, a, 16, None) == B.DGC_ERR_CAPACITY
    dec = dgc_lib.dgc_decode_accumulate
    ptrs = (C.c_void_p * 1)(a)
    cnt = (C.c_int64 * 1)(5)
    assert dec(d._h, None, 10, 1, ptrs, ptrs, cnt, None, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert dec(d._h, a, 0, 1, ptrs, ptrs, cnt, None, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    assert dec(d._h, a, 10, 65, ptrs, ptrs, cnt, None, a, 1 << 24, None) == B.DGC_ERR_CAPACITY
    neg = (C.c_int64 * 1)(-1)
    assert dec(d._h, a, 10, 1, ptrs, ptrs, neg, None, a, 1 << 24, None) == B.DGC_ERR_INVALID_ARG
    huge = (C.c_int64 * 1)(1 << 30)      # more entries than a set of 200064 elements can need
    assert dec(d._h, a, 10, 1, ptrs, ptrs, huge, None, a, 1 << 24, None) == B.DGC_ERR_CAPACITY
    odd = (C.c_void_p * 1)(a + 1)
    assert dec(d._h, a, 10, 1, odd, ptrs, cnt, None, a, 1 << 24, None) == B.DGC_ERR_ALIGNMENT
    assert dgc_lib.dgc_profile_stream_ceiling(None, a, a, 10, 0, None) == B.DGC_ERR_INVALID_ARG
    assert dgc_lib.dgc_profile_stream_ceiling(a, a, a, 10, 17, None) == B.DGC_ERR_INVALID_ARG
    assert dgc_lib.dgc_profile_stream_ceiling(a, a + 4, a, 10, 0, None) == B.DGC_ERR_ALIGNMENT
    d.close()


def test_static_entry_point_refuses_a_set_beyond_its_array(dgc_lib):
    """dgc_compress_static checks the workspace the set needs against its 8 MiB array before
    anything touches the device."""
    gs = S.speech_set()
    d = B.Dgc(B.dgc_config_default(), gs.offsets)
    assert d.dgc_workspace_bytes() > 8 << 20
    layout = d.dgc_recommended_payload_layout(0.001)
    arr = (C.c_int64 * len(layout))(*layout)
    st = dgc_lib.dgc_compress_static(d._h, 256, 256, 256, 256, 256, arr, 256, 256, 0, None)
    assert st == B.DGC_ERR_CAPACITY
    assert b"8388608" in dgc_lib.dgc_last_error_string()
    assert dgc_lib.dgc_compress_static(None, 256, 256, 256, 256, 256, arr, 256, 256, 0, None) == B.DGC_ERR_INVALID_ARG
    d.close()
