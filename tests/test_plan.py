"""Host logic: which kernels a call launches (probsparse_describe_plan), for the benchmark
workloads and for the shapes by which the GPU parity tests mean to reach each kernel.  No GPU."""
import ctypes
import math

import pytest

from paper_2106_09236_amd import binding as psa
from paper_2106_09236_amd import workloads as W
from tests import cases


ERR_NULL, ERR_SHAPE, ERR_ARG = -1, -2, -4          # psa_status_t in include/probsparse.h


def plan(B, H, L, U, dtype, c=5.0, r_sparse=None, u_stride=0):
    shape = psa.make_shape(B, H, L, U, psa.PSA_F32 if dtype == "f32" else psa.PSA_BF16)
    if u_stride:
        return psa.probsparse_describe_plan(shape, None, u_stride)
    rule, factor = (psa.U_LOG, c) if r_sparse is None else (psa.U_RATIO, r_sparse)
    return psa.probsparse_describe_plan(shape, psa.PsaOptions(rule, psa.FILL_MEAN, factor))


def of(cfg, **kw):
    return plan(cfg.B, cfg.H, cfg.L, cfg.U, cfg.dtype, cfg.c, **kw)


def test_benchmark_workloads_take_the_kernels_the_design_names():
    p = of(W.CONFIGS["tiny"])
    assert (p["measure"], p["select"], p["attend"], p["merge"]) == ("lds", "lists", "key_split", "none")
    p = of(W.CONFIGS["conformer_s"])
    assert (p["measure"], p["select"], p["lists"], p["attend"]) == ("lds", "lists", "4", "key_split")
    assert (p["u_max"], p["key_splits"], p["merge"]) == ("32", "4", "last_work_group")
    p = of(W.CONFIGS["ragged"])
    assert (p["measure"], p["select"], p["attend"], p["key_splits"], p["merge"]) == ("lds_half", "lists", "key_split", "1", "none")
    p = of(W.CONFIGS["conformer_l"])
    # streamed heads with at most 8 measure work-groups each: ranked lists, no select launch
    assert (p["measure"], p["select"], p["lists"], p["attend"], p["merge"]) == ("stream", "lists", "8", "key_split", "last_work_group")
    assert p["u_max"] == str(math.ceil(5 * math.log(2048)))
    p = of(W.CONFIGS["longform"])
    assert (p["measure"], p["select"], p["segments"], p["lists"], p["merge"]) == ("stream", "segments", "8", "8", "kernel")


def test_half_of_the_queries_kept_takes_the_rows_kernels():
    assert of(W.CONFIGS["conformer_s"], r_sparse=0.5)["attend"] == "rows_half_keys"
    assert of(W.CONFIGS["conformer_l"], r_sparse=0.5)["attend"] == "rows_half_keys"
    assert of(W.CONFIGS["ragged"], r_sparse=0.5)["attend"] == "rows_half_keys"
    assert of(W.CONFIGS["tiny"], r_sparse=0.5)["attend"] == "key_split"                 # 4 heads: too few waves
    assert plan(32, 4, 512, 32, "f32", r_sparse=0.5)["attend"] == "rows"                # 2048 waves of 16 queries
    assert plan(2, 4, 512, 32, "f32", r_sparse=0.5)["attend"] == "key_split"
    assert plan(2, 8, 2048, 40, "bf16", r_sparse=0.5)["attend"] == "key_split"          # 256 work-groups: one round


@pytest.mark.parametrize("dtype,B,H,L,r,attend", [
    # the cases of test_many_queries_many_heads
    ("bf16", 16, 8, 1024, 0.5, "rows_half_keys"), ("f32", 16, 4, 1024, 0.5, "rows"), ("bf16", 24, 4, 700, 0.75, "rows_half_keys"),
    ("f32", 16, 4, 512, 0.75, "rows_half_keys"), ("f32", 8, 8, 521, 0.75, "rows_half_keys"), ("f32", 4, 4, 512, 0.75, "rows_half_keys"),
    ("bf16", 8, 4, 1040, 0.5, "rows_half_keys"), ("bf16", 32, 4, 512, 0.75, "rows_half_keys"),
])
def test_gpu_cases_for_many_queries_reach_the_rows_kernels(dtype, B, H, L, r, attend):
    assert plan(B, H, L, 12, dtype, r_sparse=r)["attend"] == attend


@pytest.mark.parametrize("dtype,B,H,L,c,attend", [
    # the cases of test_some_dozen_queries_many_heads
    ("f32", 32, 4, 512, 12.0, "rows_half_keys"), ("bf16", 64, 4, 512, 12.0, "rows_half_keys"),
    ("bf16", 32, 4, 500, 30.0, "rows_half_keys"), ("f32", 16, 4, 500, 20.0, "rows_half_keys"),
    # a second round of work-groups, or too few waves: the keys stay split over work-groups
    ("f32", 64, 4, 512, 12.0, "key_split"), ("f32", 16, 4, 1024, 12.0, "key_split"), ("bf16", 16, 8, 2048, 12.0, "key_split"),
])
def test_gpu_cases_for_some_dozen_queries(dtype, B, H, L, c, attend):
    p = plan(B, H, L, 16, dtype, c=c)
    assert 64 <= int(p["u_max"]) < 256 and p["attend"] == attend


def test_given_index_sets():
    p = plan(16, 4, 512, 32, "f32", u_stride=32)
    assert (p["measure"], p["select"], p["attend"]) == ("none", "given_inline", "key_split")
    assert plan(16, 8, 640, 4, "f32", u_stride=560)["attend"] == "rows"
    assert plan(8, 4, 640, 4, "f32", u_stride=560)["attend"] == "rows_half_keys"
    assert plan(16, 4, 640, 4, "bf16", u_stride=560)["attend"] == "rows_half_keys"
    # index rows longer than the work-groups' list, heads of more than 4096 frames: the prep kernel
    assert plan(1, 2, 2600, 4, "bf16", u_stride=2300)["select"] == "given_prep"
    assert plan(1, 2, 4200, 4, "bf16", u_stride=300)["select"] == "given_prep"
    assert plan(1, 2, 4096, 4, "bf16", u_stride=300)["select"] == "given_inline"


def test_select_forms_by_head_length():
    assert plan(2, 2, 1024, 16, "bf16")["measure"] == "lds"
    assert plan(2, 2, 512, 16, "bf16")["measure"] == "lds_half"
    assert plan(2, 2, 512, 16, "f32")["measure"] == "lds"
    assert plan(2, 2, 513, 16, "f32")["measure"] == "stream"
    assert plan(2, 2, 2048, 16, "bf16")["select"] == "kernel"
    assert plan(2, 2, 2049, 16, "bf16")["select"] == "segments"
    assert plan(64, 8, 4096, 16, "bf16")["select"] == "kernel"          # 512 heads: no CU left for segments


def _plans(draws):
    return [plan(d["B"], d["H"], d["L"], d["U"], d["dtype"], d["c"], d["r_sparse"]) for d in draws]


def test_seeded_sweeps_cover_the_kernels_they_are_meant_to():
    short = _plans(cases.sweep_draws())
    assert {p["measure"] for p in short} == {"lds", "lds_half", "stream"}
    assert {p["select"] for p in short} >= {"lists", "kernel"}
    assert {p["merge"] for p in short} >= {"none", "last_work_group", "kernel"}
    long = _plans(cases.long_head_draws())
    assert {p["measure"] for p in long} == {"stream"}
    assert {p["select"] for p in long} == {"kernel", "segments"}
    segs = {int(p["segments"]) for p in long}
    assert 0 in segs and 8 in segs and any(2 <= s < 8 for s in segs)
    assert "kernel" in {p["merge"] for p in long}


def test_many_head_sweep_reaches_rows_kernels_and_inline_index_sets():
    seen = set()
    for d in cases.many_head_draws():
        if d["mode"] == 2:
            p = plan(d["B"], d["H"], d["L"], d["U"], d["dtype"], u_stride=d["stride"])
        else:
            p = plan(d["B"], d["H"], d["L"], d["U"], d["dtype"], d["c"])
        seen.add((p["select"], p["attend"]))
    assert ("given_inline", "key_split") in seen
    assert any(sel == "given_inline" and att != "key_split" for sel, att in seen)
    assert any(sel in ("lists", "kernel") and att == "rows_half_keys" for sel, att in seen)


def test_describe_plan_argument_errors():
    lib = psa.load()
    shape = psa.make_shape(1, 1, 64, 8, psa.PSA_F32)
    opt = psa.PsaOptions(psa.U_LOG, psa.FILL_MEAN, 5.0)
    buf = ctypes.create_string_buffer(512)
    tiny = ctypes.create_string_buffer(8)
    f = lib.probsparse_describe_plan
    assert f(None, ctypes.byref(opt), 0, buf, 512) == ERR_NULL
    assert f(ctypes.byref(shape), None, 0, buf, 512) == ERR_NULL
    assert f(ctypes.byref(shape), ctypes.byref(opt), 0, None, 512) == ERR_NULL
    assert f(ctypes.byref(shape), ctypes.byref(opt), 0, tiny, 8) == ERR_ARG
    assert f(ctypes.byref(shape), ctypes.byref(opt), -1, buf, 512) == ERR_ARG
    assert f(ctypes.byref(shape), None, 65, buf, 512) == ERR_ARG            # stride beyond L
    bad = psa.PsaOptions(psa.U_LOG, psa.FILL_MEAN, -1.0)
    assert f(ctypes.byref(shape), ctypes.byref(bad), 0, buf, 512) == ERR_ARG
    wrong = psa.make_shape(1, 1, 64, 8, psa.PSA_F32, D=32)
    assert f(ctypes.byref(wrong), ctypes.byref(opt), 0, buf, 512) == ERR_SHAPE
    assert f(ctypes.byref(shape), ctypes.byref(opt), 0, buf, 512) == 0 and b"measure=lds" in buf.value
