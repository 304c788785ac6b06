"""Host-side tests of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2308_15030_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a non-null, 256-byte aligned "device pointer" that is never dereferenced


def test_exports_match_header():
    import glob
    text = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(smoe_[a-z_]+)\s*\(", text))
    assert declared == set(b.EXPORTS)
    lib = C.CDLL(b.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    for six in ("smoe_route", "smoe_importance", "smoe_permute", "smoe_expert_ffn", "smoe_combine",
                "smoe_set_resident"):
        assert six in declared


def _status(fn, *a):
    with pytest.raises(b.SmoeError) as e:
        fn(*a)
    assert b.smoe_last_error() != ""
    return e.value.status


def test_create_validation():
    ok = dict(E=8, K=2, d_model=64, d_ff=256, max_tokens=256, dtype=b.SMOE_F32)
    h = b.smoe_create(**ok)
    assert b.smoe_workspace_bytes(h) > 256 * 256 * 4
    assert b.smoe_slot_weight_bytes(h) == 2 * 64 * 256 * 4
    b.smoe_destroy(h)
    for bad in (dict(E=0), dict(E=257), dict(K=0), dict(K=9), dict(d_model=0), dict(d_ff=-4),
                dict(max_tokens=0), dict(dtype=7), dict(gate_mode=2), dict(d_model=66),
                dict(dtype=b.SMOE_BF16, d_model=48)):
        assert _status(lambda kw: b.smoe_create(**kw), {**ok, **bad}) == b.SMOE_EINVAL
    assert b._lib.smoe_create(None, None) == b.SMOE_EINVAL
    assert b._lib.smoe_destroy(None) == b.SMOE_EINVAL
    assert b.smoe_workspace_bytes(None) == 0


def test_workspace_grows_with_tokens():
    a = b.smoe_create(64, 16, 768, 3072, 4096, b.SMOE_BF16)
    c = b.smoe_create(64, 16, 768, 3072, 8192, b.SMOE_BF16)
    assert b.smoe_workspace_bytes(c) > b.smoe_workspace_bytes(a) >= 4096 * 3072 * 2
    assert b.smoe_slot_weight_bytes(a) == 16 * 768 * 3072 * 2
    b.smoe_destroy(a); b.smoe_destroy(c)


def test_state_and_argument_errors_before_any_launch():
    h = b.smoe_create(8, 2, 64, 256, 128, b.SMOE_F32)
    lib = b._lib
    # nothing bound yet
    assert lib.smoe_route(h, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_ESTATE
    assert lib.smoe_set_resident(h, 0, 0, FAKE, FAKE, None) == b.SMOE_ESTATE
    # bind: nulls and alignment
    assert lib.smoe_bind(h, None, FAKE, FAKE, FAKE, FAKE) == b.SMOE_EINVAL
    assert lib.smoe_bind(h, FAKE, FAKE + 64, FAKE, FAKE, FAKE) == b.SMOE_EINVAL
    assert lib.smoe_bind(h, FAKE, FAKE, FAKE, FAKE, FAKE) == b.SMOE_OK
    # set_resident ranges
    assert lib.smoe_set_resident(h, -1, 0, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_set_resident(h, 2, 0, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_set_resident(h, 0, 8, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_set_resident(h, 0, 0, None, FAKE, None) == b.SMOE_EINVAL
    assert "null" in b.smoe_last_error()
    # slots not all filled -> route / ffn refuse; T range is checked first
    assert lib.smoe_route(h, FAKE, 129, FAKE, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_route(h, FAKE, -1, FAKE, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_route(h, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_ESTATE
    assert lib.smoe_expert_ffn(h, FAKE, FAKE, 4, FAKE, None) == b.SMOE_ESTATE
    assert "slots" in b.smoe_last_error()
    # null buffers and flags on the calls that do not need a full resident set
    assert lib.smoe_importance(h, None, FAKE, FAKE, 4, FAKE, FAKE, FAKE, 0, None) == b.SMOE_EINVAL
    assert lib.smoe_importance(h, FAKE, FAKE, FAKE, 4, FAKE, FAKE, FAKE, 2, None) == b.SMOE_EINVAL
    assert lib.smoe_importance(h, FAKE, FAKE, FAKE, 4, None, FAKE, FAKE, 0, None) == b.SMOE_EINVAL
    assert lib.smoe_permute(h, FAKE, None, 4, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_permute(h, FAKE, FAKE, 4, FAKE, FAKE, FAKE, None, None) == b.SMOE_EINVAL
    assert lib.smoe_permute(h, FAKE + 4, FAKE, 4, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_combine(h, FAKE, FAKE, None, None, 4, FAKE, None) == b.SMOE_EINVAL
    assert lib.smoe_combine(h, FAKE, FAKE, FAKE, None, 999, FAKE, None) == b.SMOE_EINVAL
    # legal no-ops
    assert lib.smoe_combine(h, None, None, None, None, 0, None, None) == b.SMOE_OK
    assert lib.smoe_importance(h, None, None, None, 0, FAKE, FAKE, FAKE, 1, None) == b.SMOE_OK
    assert lib.smoe_route(None, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == b.SMOE_EINVAL
    b.smoe_destroy(h)


def test_maps_and_policy_on_host():
    h = b.smoe_create(6, 3, 64, 64, 16, b.SMOE_F32)
    s2e = np.zeros(3, np.int32); e2s = np.zeros(6, np.int32)
    b.smoe_get_maps(h, s2e, e2s)
    assert (s2e == -1).all() and (e2s == -1).all()
    # empty slots: the three best experts fill slots 0,1,2 in descending score order
    score = np.array([0.1, 0.9, 0.3, 0.9, 0.0, 0.5], np.float32)
    cs = np.empty(3, np.int32); ce = np.empty(3, np.int32)
    n = b.smoe_select_resident(h, score, cs, ce)
    assert n == 3 and cs.tolist() == [0, 1, 2] and ce.tolist() == [1, 3, 5]
    assert b._lib.smoe_select_resident(h, None, cs.ctypes.data, ce.ctypes.data) == b.SMOE_EINVAL
    b.smoe_destroy(h)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 on its own."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    for header in ("swapmoe.h", "swapmoe_profile.h"):
        r = subprocess.run([gcc, "-x", "c", "-std=c99", "-fsyntax-only", "-Wall", "-Werror", "-I",
                            os.path.join(ROOT, "include"), os.path.join(ROOT, "include", header)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_spare_slots_and_async_calls_without_a_gpu():
    h = b.smoe_create(8, 2, 64, 256, 128, b.SMOE_BF16, spare_slots=2)
    assert b.smoe_slot_weight_bytes(h) == (2 + 2) * 64 * 256 * 2
    base = b.smoe_create(8, 2, 64, 256, 128, b.SMOE_BF16)
    # staging area for host-bank loads: one expert (two matrices) per spare slot
    assert b.smoe_workspace_bytes(h) - b.smoe_workspace_bytes(base) >= 2 * 2 * 64 * 256 * 2
    assert _status(lambda: b.smoe_create(8, 2, 64, 256, 128, b.SMOE_BF16, spare_slots=9)) == b.SMOE_EINVAL
    score = np.zeros(8, np.float32)
    assert _status(b.smoe_update_begin, h, score) == b.SMOE_ESTATE          # not bound
    assert _status(b.smoe_update_begin, base, score) == b.SMOE_ESTATE
    assert b._lib.smoe_update_tick(h, FAKE, FAKE, None, None) == b.SMOE_ESTATE
    assert b._lib.smoe_update_pending(None) == b.SMOE_EINVAL
    assert b.smoe_update_pending(h) == 0
    b.smoe_destroy(h); b.smoe_destroy(base)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_policy_unit_on_host():
    """Rankings and the load-on-miss plan are host code: checked here without a GPU."""
    count = np.array([5, 0, 9, 9, 1, 2], np.int32)
    score = np.array([0.5, 0.0, 2.0, 0.1, 3.0, 0.2], np.float32)
    en = np.array([1.0, 6.0, 2.0, 5.0, 3.0, 4.0], np.float32)
    rank = np.empty(6, np.float32)
    for policy, src in ((b.SMOE_POLICY_IMPORTANCE, score), (b.SMOE_POLICY_COUNT, count), (b.SMOE_POLICY_MAGNITUDE, en)):
        b.smoe_policy_scores(policy, 6, count, score, en, rank)
        assert np.array_equal(rank, src.astype(np.float32))
    assert _status(b.smoe_policy_scores, 3, 6, count, score, en, rank) == b.SMOE_EINVAL
    assert _status(b.smoe_policy_scores, b.SMOE_POLICY_COUNT, 6, None, score, en, rank) == b.SMOE_EINVAL
    # load on miss on a handle whose slots are all empty: the most requested experts fill slots 0, 1, 2
    h = b.smoe_create(7, 3, 64, 64, 16, b.SMOE_F32)
    cs = np.empty(3, np.int32); ce = np.empty(3, np.int32)
    oe = np.array([3, 4, 5, 6, 6], np.int32)
    n = b.smoe_on_demand_plan(h, oe, 5, cs, ce)
    assert n == 3 and cs.tolist() == [0, 1, 2] and ce.tolist() == [6, 3, 4]
    # the plan changes no map (the caller loads): the same batch again asks for the same loads
    assert b.smoe_on_demand_plan(h, oe, 5, cs, ce) == 3 and ce.tolist() == [6, 3, 4]
    assert b.smoe_on_demand_plan(h, oe, 0, cs, ce) == 0          # an empty batch asks for nothing
    assert _status(b.smoe_on_demand_plan, h, np.array([9], np.int32), 1, cs, ce) == b.SMOE_EINVAL
    b.smoe_destroy(h)


def test_profile_bookkeeping_on_host():
    """E_memory from the shape alone, and the update-period search on a measured-looking sweep."""
    m = b.smoe_profile_memory(64, 16, 768, 3072, 32, b.SMOE_BF16, spare_slots=1)
    per = 2 * 768 * 3072 * 2
    assert m["expert_bytes"] == per and m["resident_bytes"] == 17 * per and m["bank_bytes"] == 64 * per
    assert m["router_bytes"] == 64 * 768 * 4
    h = b.smoe_create(64, 16, 768, 3072, 32, b.SMOE_BF16, spare_slots=1)
    assert m["workspace_bytes"] == b.smoe_workspace_bytes(h) and b.smoe_slot_weight_bytes(h) * 2 == m["resident_bytes"]
    b.smoe_destroy(h)
    with pytest.raises(b.SmoeError):
        b.smoe_profile_memory(64, 65, 768, 3072, 32, b.SMOE_BF16)
    # step latency against update frequency, lowest frequency (longest period) first: flat, then it rises
    periods = [128, 64, 32, 16, 8, 4, 2]
    lat = [40.7, 41.4, 42.7, 44.4, 48.5, 59.8, 83.3]
    assert periods[b.smoe_period_inflection(lat, 0.10)] == 16   # 48.5 is the first point above 1.1 x 40.7
    assert periods[b.smoe_period_inflection(lat, 0.03)] == 64   # 42.7 > 1.03 x 40.7
    assert periods[b.smoe_period_inflection(lat, 2.0)] == 2     # never rises that much: the whole sweep is flat
    assert b.smoe_period_inflection([50.0, 45.0, 44.0, 49.0], 0.10) == 2   # the floor follows the minimum so far
    assert b.smoe_period_inflection([7.0], 0.1) == 0
    with pytest.raises(b.SmoeError):
        b.smoe_period_inflection([], 0.1)
    # the event bracket refuses an end without a begin, before any HIP call
    h = b.smoe_create(8, 2, 64, 256, 128, b.SMOE_F32)
    us = C.c_float()
    assert b._lib.smoe_profile_end(h, None, C.byref(us)) == b.SMOE_ESTATE
    b.smoe_destroy(h)
