"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its host-only entry points (shape validation, keep count, refresh
schedule, status strings) behave as documented."""

import ctypes
import json
import os
import re

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20813_amd import pulsecol as pc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pulsecol.h")


def _declared():
    src = open(HEADER).read()
    return sorted(set(re.findall(r"PULSECOL_API\s+[\w\s\*]+?\b(pulsecol_\w+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 13
    assert sorted(pc.EXPORTS) == names
    L = ctypes.CDLL(pc.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    seen = {pc.status_str(i) for i in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert pc.status_str(99) == "unknown status"


@pytest.mark.parametrize("kw,want", [
    (dict(), pc.OK),
    (dict(batch=0), pc.ERR_INVALID_ARG),
    (dict(heads=0), pc.ERR_INVALID_ARG),
    (dict(seq=0), pc.ERR_INVALID_ARG),
    (dict(head_dim=96), pc.ERR_UNSUPPORTED),
    (dict(head_dim=256), pc.ERR_UNSUPPORTED),
    (dict(group_size=-1), pc.ERR_INVALID_ARG),
    (dict(group_size=32), pc.OK),                       # the paper's group sizes: small-group kernel
    (dict(group_size=384), pc.OK),
    (dict(group_size=48), pc.ERR_UNSUPPORTED),          # groups are whole blocks of 32 queries
    (dict(group_size=64, dtype=pc.F32), pc.ERR_UNSUPPORTED),   # f32 query blocks are 128 rows
    (dict(group_size=512), pc.OK),                      # 8 groups of two query blocks
    (dict(kv_heads=8), pc.OK),                          # grouped-query layout: 4 query heads per K/V head
    (dict(kv_heads=5), pc.ERR_INVALID_ARG),             # not a divisor of heads
    (dict(kv_heads=64), pc.ERR_INVALID_ARG),
    (dict(kv_heads=-1), pc.ERR_INVALID_ARG),
    (dict(kv_heads=8, kv_strides=(0, 0, 100)), pc.ERR_INVALID_ARG),    # K/V row stride below head_dim
    (dict(kv_heads=8, kv_strides=(0, 0, 132)), pc.ERR_ALIGNMENT),
    (dict(group_size=4096), pc.OK),                     # one group covering every query == per head
    (dict(strides=(0, 0, 100)), pc.ERR_INVALID_ARG),    # stride_n < head_dim
    (dict(strides=(0, 0, 132)), pc.ERR_ALIGNMENT),      # not a multiple of 8 bf16 elements
    (dict(strides=(0, 0, 136)), pc.OK),
    (dict(scale=-1.0), pc.ERR_INVALID_ARG),
    (dict(scale=float("nan")), pc.ERR_INVALID_ARG),
    # the kernels address a head's rows with 32-bit byte offsets formed by 24-bit multiplies
    (dict(seq=1 << 23), pc.OK),                                         # 8M rows x 256 B = 2 GiB per head
    (dict(seq=1 << 24), pc.ERR_UNSUPPORTED),                            # row number needs 25 bits
    (dict(seq=1 << 20, strides=(0, 0, 2040)), pc.OK),                   # just under 4 GiB per head
    (dict(seq=1 << 20, strides=(0, 0, 2048)), pc.ERR_UNSUPPORTED),      # 4 GiB per head
    (dict(seq=64, strides=(0, 0, 1 << 23)), pc.ERR_UNSUPPORTED),        # row stride of 2^24 bytes
    (dict(seq=1 << 20, kv_heads=8, kv_strides=(0, 0, 2048)), pc.ERR_UNSUPPORTED),
])
def test_validate_shape(kw, want):
    args = dict(batch=1, heads=32, seq=4096, head_dim=128, dtype=pc.BF16, group_size=0, strides=(0, 0, 0), scale=0.0)
    args.update(kw)
    assert pc.validate_shape(pc.make_shape(**args)) == want
    if want != pc.OK:
        assert pc.last_error(None)


def test_validate_shape_dtype_and_null():
    s = pc.make_shape(1, 2, 256, 64, pc.F32)
    assert pc.validate_shape(s) == pc.OK
    s.dtype = 7
    assert pc.validate_shape(s) == pc.ERR_UNSUPPORTED
    assert pc.lib().pulsecol_validate_shape(None) == pc.ERR_INVALID_ARG
    s4 = pc.make_shape(1, 2, 256, 64, pc.F32, strides=(0, 0, 66))
    assert pc.validate_shape(s4) == pc.ERR_ALIGNMENT


def test_num_keep_matches_the_oracle_rule():
    for n, r in ((256, .25), (4096, .1), (16384, .1), (32768, .05), (32768, .1), (32768, .2), (65536, .1),
                 (100, .29), (5, .1), (7, 1.0), (1000, 0.333), (3, 0.5)):
        assert pc.num_keep(n, r) == oracle.num_keep(n, r), (n, r)
    assert pc.num_keep(0, .5) == -1 and pc.num_keep(8, 0.0) == -1 and pc.num_keep(8, 1.01) == -1
    assert pc.num_keep(8, float("nan")) == -1


def test_num_keep_sweep_over_decimal_ratios():
    """Every ratio with one to four decimal digits at the workloads' context lengths (and a few
    lengths that are not powers of two): the library's floating-point floor against the oracle's
    exact rational one (Sec. 3.1, sparsity-budget constraint)."""
    from fractions import Fraction
    L = pc.lib()
    lengths = (256, 4096, 16384, 32768, 65536, 131072, 1000, 777, 12345)
    bad = []
    for digits in (1, 2, 3, 4):
        den = 10 ** digits
        for num in range(1, den + 1):
            r = num / den
            for n in lengths:
                want = max(1, (Fraction(num, den) * n).__floor__())
                got = L.pulsecol_num_keep(n, r)
                if got != want:
                    bad.append((n, r, got, want))
    assert not bad, bad[:10]
    # the oracle's own rule on a sample of the same grid (it reads the ratio as the decimal written)
    for num in range(1, 10001, 37):
        for n in (4096, 65536, 777):
            assert oracle.num_keep(n, num / 10000) == max(1, (Fraction(num, 10000) * n).__floor__())


def test_max_keep_ratio_is_validated():
    args = dict(batch=1, heads=2, seq=512, head_dim=128, dtype=pc.BF16)
    assert pc.validate_shape(pc.make_shape(**args, max_keep_ratio=0.25)) == pc.OK
    assert pc.validate_shape(pc.make_shape(**args, max_keep_ratio=1.0)) == pc.OK
    assert pc.validate_shape(pc.make_shape(**args, max_keep_ratio=1.5)) == pc.ERR_INVALID_ARG
    assert pc.validate_shape(pc.make_shape(**args, max_keep_ratio=-0.1)) == pc.ERR_INVALID_ARG
    assert pc.validate_shape(pc.make_shape(**args, max_keep_ratio=float("nan"))) == pc.ERR_INVALID_ARG


def test_refresh_schedule_matches_golden_and_oracle():
    with open(os.path.join(ROOT, "tests", "golden", "eq8_schedules.json")) as f:
        for c in json.load(f)["cases"]:
            assert pc.refresh_schedule(c["T"], c["eta"], c["R"]) == c["tau"]
    for T, eta, R in ((100, .5, 7), (1000, .3, 16), (17, 1.0, 17), (50, .1, 3), (100, .29, 5), (3, .1, 2)):
        assert pc.refresh_schedule(T, eta, R) == oracle.refresh_schedule(T, eta, R)
    with pytest.raises(pc.PulseColError):
        pc.refresh_schedule(0, .3, 4)
    with pytest.raises(pc.PulseColError):
        pc.refresh_schedule(10, 1.5, 4)


def test_schedule_variants_match_golden_and_oracle():
    with open(os.path.join(ROOT, "tests", "golden", "schedule_variants.json")) as f:
        g = json.load(f)
    for c in g["power"]:
        assert pc.refresh_schedule_power(c["T"], c["eta"], c["R"]) == c["tau"]
    for c in g["random"]:
        assert pc.refresh_schedule_random(c["T"], c["eta"], c["R"], c["uniforms"]) == c["tau"]
    rng = np.random.default_rng(11)
    for T, eta, R in ((100, .5, 7), (1000, .3, 16), (17, 1.0, 17), (50, .1, 3), (100, .29, 5), (1024, .3, 64)):
        assert pc.refresh_schedule_power(T, eta, R) == oracle.refresh_schedule_power(T, eta, R)
        u = rng.random(R - 1).tolist()
        assert pc.refresh_schedule_random(T, eta, R, u) == oracle.refresh_schedule_random(T, eta, R, u)
    for bad in ((10, .3, 5, [.1, .2, .3, .4]), (10, 1.0, 3, [.5, 1.0]), (10, 1.0, 3, [-.1, .2]), (0, .5, 2, [.5])):
        with pytest.raises(pc.PulseColError):
            pc.refresh_schedule_random(*bad)
    with pytest.raises(pc.PulseColError):
        pc.refresh_schedule_power(10, 0.0, 3)


def test_schedule_driver_steps():
    from paper_2605_20813_amd import schedule as sch
    assert sch.refresh_steps(1024, .3, 4) == [0, 102, 204, 306]
    assert sch.refresh_steps(110, .3, 3) == [0, 16, 32]
    assert sch.refresh_steps(100, .3, 4, "power") == [0, 3, 12, 29]
    assert sch.refresh_steps(20, .5, 4, "random", [0.0, 0.5, 0.99]) == [0, 1, 6, 9]
    assert sch.refresh_steps(128, .3, 8, "power") == [0, 3, 6, 12, 18, 27, 37]      # a repeated step counts once
    with pytest.raises(ValueError):
        sch.refresh_steps(10, .5, 2, "random")
    with pytest.raises(ValueError):
        sch.refresh_steps(10, .5, 2, "sometimes")


def test_null_context_calls_fail_cleanly():
    L = pc.lib()
    assert L.pulsecol_attn(None, None, None, None, None, 1, None, None) == pc.ERR_INVALID_ARG
    assert L.pulsecol_select(None, None, None, 0.1, 1, None, None) == pc.ERR_INVALID_ARG
    assert L.pulsecol_scores(None, None, None, None, None) == pc.ERR_INVALID_ARG
    assert L.pulsecol_topk(None, None, 1, None, None) == pc.ERR_INVALID_ARG
    assert L.pulsecol_attn_dense(None, None, None, None, None, None, None) == pc.ERR_INVALID_ARG
    assert L.pulsecol_destroy(None) == pc.OK
    assert L.pulsecol_create(None, None, 0) == pc.ERR_INVALID_ARG


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful on a box without a GPU")
def test_create_without_gpu_reports_an_error():
    with pytest.raises(pc.PulseColError):
        pc.Context(1, 2, 256, 64, pc.F32)
