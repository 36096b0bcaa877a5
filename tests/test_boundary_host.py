"""CPU-only tests of the boundary: the shared library loads and exports every symbol that
include/hs.h declares, and its host-only logic (admission control of Section IV-A, latency
determinism metrics of Section V-A, description validation, workspace sizing) behaves as
documented.  No compute call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2402_04466_amd as hs
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hs.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(hs_[a-z_]+)\s*\(", header))
    assert {"hs_create_app", "hs_submit_frame", "hs_poll_result", "hs_set_partition"} <= names
    lib = ctypes.CDLL(hs.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), f"libhs.so does not export {n}"
    assert "gfx950" in hs.hs_version()


def test_binding_struct_sizes_match_the_header(tmp_path):
    src = tmp_path / "sz.c"
    src.write_text('#include <stdio.h>\n#include "hs.h"\nint main(void){printf("%zu %zu %zu %zu\\n",'
                   "sizeof(hs_app_desc),sizeof(hs_result),sizeof(hs_latency_metrics),"
                   "sizeof(hs_kernel_time));printf(\"%zu %zu\\n\",sizeof(hs_feed),sizeof(hs_mwu));"
                   "return 0;}\n")
    exe = tmp_path / "sz"
    import subprocess
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    want = [int(v) for v in subprocess.check_output([str(exe)]).split()]
    from paper_2402_04466_amd import api
    got = [ctypes.sizeof(c) for c in (hs.hs_app_desc, hs.hs_result, hs.hs_latency_metrics,
                                      hs.hs_kernel_time, hs.hs_feed, api.hs_mwu)]
    assert got == want


def test_stream_driver_and_group_calls_reject_bad_arguments_without_a_gpu():
    """Argument checks come before any GPU work, so they can be exercised here."""
    from paper_2402_04466_amd import api
    lib = api.load()
    assert lib.hs_run_feeds(None, 1, 60.0, 10, None, None, None, None) == hs.HS_E_INVAL
    feeds = (hs.hs_feed * 1)()                       # all-zero feed: no application, no buffers
    res = (ctypes.c_void_p * 1)()
    assert lib.hs_run_feeds(feeds, 1, 60.0, 10, res, None, None, None) == hs.HS_E_INVAL
    assert "feed 0" in hs.hs_last_error()
    assert lib.hs_run_feeds(feeds, 1, -1.0, 10, res, None, None, None) == hs.HS_E_INVAL
    assert lib.hs_run_feeds(feeds, 0, 60.0, 10, res, None, None, None) == hs.HS_E_INVAL
    out = ctypes.c_void_p()
    assert lib.hs_create_group(None, None, 2, ctypes.byref(out)) == hs.HS_E_INVAL
    assert lib.hs_destroy_group(None) == hs.HS_E_INVAL
    assert lib.hs_submit_group(None, None, None, 0) == hs.HS_E_INVAL
    assert lib.hs_poll_group(None, None) == hs.HS_E_INVAL
    assert lib.hs_wait_group(None, None, 0) == hs.HS_E_INVAL
    mux = ctypes.c_void_p()
    assert lib.hs_create_mux(None, 3, ctypes.byref(mux)) == hs.HS_E_INVAL
    assert lib.hs_destroy_mux(None) == hs.HS_E_INVAL
    assert lib.hs_mux_submit(None, 0, None, None, 0) == hs.HS_E_INVAL
    assert lib.hs_mux_poll(None, 0, None) == hs.HS_E_INVAL
    assert lib.hs_mux_wait(None, 0, None, 0) == hs.HS_E_INVAL
    assert lib.hs_submit_batch_after(None, None, None, 0, None) == hs.HS_E_INVAL
    sec = ctypes.c_double()
    assert lib.hs_partition_copy(None, None, None, 16, 1, ctypes.byref(sec)) == hs.HS_E_INVAL


# ---- admission control ---------------------------------------------------------------------
def _m(cus):
    return hs.cu_mask_words(cus)


def test_admission_disjoint_partitions_are_admitted_until_full():
    """Six equal partitions of 40 CUs (five groups of 8 consecutive CUs: 32 for inference, 8 for
    the overlay; 6 x 40 = 240 <= 256) fit; a request that touches a claimed CU does not; the two
    groups left over do."""
    claimed = np.zeros(8, np.uint32)
    for i in range(6):
        infer, over = _m(range(40 * i, 40 * i + 32)), _m(range(40 * i + 32, 40 * i + 40))
        assert hs.hs_admission_check(claimed, infer, over, 256) == hs.HS_OK
        claimed |= infer | over
    assert hs.hs_admission_check(claimed, _m(range(232, 248)), _m(range(232, 248)), 256) \
        == hs.HS_E_OVERSUBSCRIBED
    assert hs.hs_admission_check(claimed, _m(range(240, 256)), _m(range(240, 248)), 256) == hs.HS_OK


def test_admission_five_quarters_oversubscribe():
    """5 x 25 % = 125 % is the bad case named in the paper's appendix: the fifth is refused."""
    claimed = np.zeros(8, np.uint32)
    results = []
    for i in range(5):
        cus = [c % 256 for c in range(64 * i, 64 * i + 64)]
        st = hs.hs_admission_check(claimed, _m(cus), _m(cus), 256)
        results.append(st)
        if st == hs.HS_OK:
            claimed |= _m(cus)
    assert results == [hs.HS_OK] * 4 + [hs.HS_E_OVERSUBSCRIBED]


def test_admission_rejects_empty_out_of_range_and_bad_args():
    # a device of 24 CUs has a single XCD: only the emptiness / range / claim rules act
    z = np.zeros(8, np.uint32)
    assert hs.hs_admission_check(None, z, _m([1]), 24) == hs.HS_E_OVERSUBSCRIBED
    assert hs.hs_admission_check(None, _m([1]), z, 24) == hs.HS_E_OVERSUBSCRIBED
    assert hs.hs_admission_check(None, _m([24]), _m([3]), 24) == hs.HS_E_OVERSUBSCRIBED
    assert hs.hs_admission_check(None, _m([200]), _m([3]), 24) == hs.HS_E_OVERSUBSCRIBED
    assert hs.hs_admission_check(None, _m([23]), _m([3]), 24) == hs.HS_OK
    assert hs.hs_admission_check(None, _m([3]), _m([3]), 0) == hs.HS_E_INVAL
    assert "CU" in hs.hs_last_error() or "argument" in hs.hs_last_error()
    # inference and overlay masks of ONE application may overlap each other
    assert hs.hs_admission_check(z, _m(range(0, 32)), _m(range(16, 48)), 256) == hs.HS_OK


def test_admission_needs_a_cu_on_every_xcd():
    """CU i sits on XCD i mod 8 of a 256-CU device (i mod 4 with 128 CUs): a mask that leaves an
    XCD without a CU is refused with HS_E_INVAL, whichever of the two masks it is; the other
    rules are judged first."""
    full = _m(range(0, 8))
    for hole in range(8):
        cus = [c for c in range(16, 48) if c % 8 != hole]          # 28 CUs, none on XCD `hole`
        assert hs.hs_admission_check(None, _m(cus), full, 256) == hs.HS_E_INVAL
        assert f"XCD {hole}" in hs.hs_last_error() and "inference" in hs.hs_last_error()
        assert hs.hs_admission_check(None, full, _m(cus), 256) == hs.HS_E_INVAL
        assert "overlay" in hs.hs_last_error()
        assert hs.hs_admission_check(None, _m(cus + [hole + 48]), full, 256) == hs.HS_OK
    # one CU per XCD is the smallest admissible mask; they need not be consecutive
    assert hs.hs_admission_check(None, _m([0, 9, 18, 27, 36, 45, 54, 63]), full, 256) == hs.HS_OK
    assert hs.hs_admission_check(None, _m(range(0, 7)), full, 256) == hs.HS_E_INVAL
    # 128 CUs: four XCDs
    assert hs.hs_admission_check(None, _m([4, 5, 6, 7]), _m([0, 1, 2, 3]), 128) == hs.HS_OK
    assert hs.hs_admission_check(None, _m([4, 5, 6]), _m([0, 1, 2, 3]), 128) == hs.HS_E_INVAL
    # a claimed CU is reported as over-subscription even when the mask is also XCD-incomplete
    assert hs.hs_admission_check(_m([3]), _m([3]), full, 256) == hs.HS_E_OVERSUBSCRIBED


# ---- metrics ---------------------------------------------------------------------------------
def test_metrics_match_oracle_and_golden():
    x = np.random.default_rng(0).gamma(2.0, 3.0, 1000)
    for trim in (False, True):
        got, want = hs.hs_latency_metrics_compute(x, trim), oracle.determinism_metrics(x, trim)
        assert got["n"] == want["n"]
        for k in ("mean", "max", "std", "p50", "p99", "tail", "flatness"):
            assert abs(got[k] - want[k]) <= 1e-12 * max(1.0, abs(want[k])), k
    m = hs.hs_latency_metrics_compute(np.arange(1, 102), trim=False)
    assert (m["p50"], m["tail"], m["flatness"], m["max"]) == (51.0, 5.0, 80.0, 101.0)
    short = hs.hs_latency_metrics_compute([5, 1, 2, 3, 4, 1.5, 2.5, 9], trim=True)
    assert short["n"] == 6 and short["max"] == 4.0
    with pytest.raises(hs.HsError):
        hs.hs_latency_metrics_compute([], trim=True)


# ---- description validation and workspace sizing ---------------------------------------------
def _desc(**over):
    kw = dict(frame_w=1920, frame_h=1080, net_w=854, net_h=480, net=hs.HS_NET_RESNET18_CONVLSTM,
              weights=np.zeros(4, np.float32), palette=si.DEFAULT_PALETTE, frame_pitch=5760)
    kw.update(over)
    return hs.make_desc(**kw)


def test_workspace_query_and_validation():
    big = hs.hs_query_workspace(_desc())
    # fp16 weights 36.5 MB + stem output 13.1 MB + 4 activation buffers + split-K scratch ...
    assert 60e6 < big < 120e6
    assert hs.hs_query_workspace(_desc(queue_depth=4)) > big
    small = hs.hs_query_workspace(_desc(frame_w=320, frame_h=240, net_w=128, net_h=128,
                                        net=hs.HS_NET_TINY4, frame_pitch=960))
    assert small < 4e6
    for bad in (dict(frame_pitch=5761), dict(frame_pitch=100), dict(net=7), dict(queue_depth=0),
                dict(threshold=1.0), dict(alpha=1.5), dict(std=0.0), dict(net_w=0),
                dict(net_w=16000, net_h=16000)):
        with pytest.raises(hs.HsError) as ei:
            hs.hs_query_workspace(_desc(**bad))
        assert ei.value.status == hs.HS_E_INVAL, bad


def test_no_gpu_means_loud_failure_not_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(hs.HsError) as ei:
        hs.hs_init(0)
    assert ei.value.status == hs.HS_E_DEVICE


def test_mann_whitney_matches_oracle_and_rejects_empty(hs):
    """hs_mann_whitney_u (rank sums with mid-ranks) against the oracle's pairwise definition."""
    import oracle
    rng = np.random.default_rng(11)
    for n, m, shift, quant in ((30, 45, 0.0, None), (200, 150, 0.2, None), (120, 120, 0.05, 0.02),
                               (7, 5, 2.0, 0.5), (4, 4, 0.0, 1.0)):
        a = rng.normal(1.0 + shift, 0.25, n)
        b = rng.normal(1.0, 0.25, m)
        if quant:
            a, b = np.round(a / quant) * quant, np.round(b / quant) * quant
        got, ref = hs.hs_mann_whitney_u(a, b), oracle.mann_whitney_z(a, b)
        assert got["u"] == ref["u"]
        assert abs(got["z"] - ref["z"]) <= 1e-12 * max(1.0, abs(ref["z"]))
        assert got["significant"] == ref["significant"]
    same = hs.hs_mann_whitney_u([3.0, 3.0, 3.0], [3.0, 3.0])
    assert same["u"] == 3.0 and same["z"] == 0.0 and not same["significant"]
    with pytest.raises(hs.HsError):
        hs.hs_mann_whitney_u([], [1.0])


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more must exit with a message, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_seeded_inputs_hash_to_the_recorded_values():
    """The generators behind every benchmark configuration still produce the recorded bytes."""
    import importlib.util
    path = os.path.join(ROOT, "tests", "golden", "make_input_hashes.py")
    spec = importlib.util.spec_from_file_location("make_input_hashes", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = [l.rstrip("\n") for l in open(os.path.join(ROOT, "tests", "golden", "input_hashes.txt"))
            if not l.startswith("#")]
    assert list(mod.lines()) == want
