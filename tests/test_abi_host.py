"""Host-side checks of the C ABI (no GPU): the library loads, exports every
symbol the header declares, validates arguments before touching the device, and
its offline calibration agrees with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2408_07092_amd as ds
from oracle import ds_oracle as O
from workloads import WORKLOADS, make_calibration_numpy, outlier_channels

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ds_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ds_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    names = declared_functions()
    assert "ds_sparse_decode" in names and "ds_calibrate_channels" in names and len(names) >= 15
    lib = ds.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in ds_attn.h but not exported"
    assert sorted(ds.binding.EXPORTS) == names
    assert ds.ds_version() >= 100


def test_strerror_covers_all_codes():
    msgs = {ds.strerror(c) for c in range(0, -7, -1)}
    assert len(msgs) == 7 and all(msgs)
    assert ds.strerror(-99) == "unknown status"


def test_workspace_bytes_is_pure_and_monotone():
    a = ds.ds_workspace_bytes(ds.shape(1, 32, 32, 128, 4096, 4096, 8, 256))
    b = ds.ds_workspace_bytes(ds.shape(1, 32, 32, 128, 65536, 65536, 8, 4096))
    assert 0 < a < b
    assert a == ds.ds_workspace_bytes(ds.shape(1, 32, 32, 128, 4096, 4096, 8, 256))
    for bad in [ds.shape(1, 32, 32, 64, 4096, 4096, 8, 256),      # d != 128
                ds.shape(1, 32, 5, 128, 4096, 4096, 8, 256),       # Hq % Hkv
                ds.shape(1, 32, 32, 128, 5000, 4096, 8, 256),      # L > L_max
                ds.shape(0, 32, 32, 128, 4096, 4096, 8, 256)]:
        assert ds.ds_workspace_bytes(bad) == 0
    assert ds.lib().ds_workspace_bytes(None) == 0


FAKE = ctypes.c_void_p(0x10000)   # aligned, never dereferenced: validation fails first


def _sparse(shape, q=FAKE, label=FAKE, K=FAKE, V=FAKE, ch=FAKE, out=FAKE, idx=None, ws=FAKE, ws_bytes=1 << 40):
    return ds.lib().ds_sparse_decode(q, label, K, V, ch, out, idx, ws, ws_bytes,
                                     ctypes.byref(shape) if shape is not None else None, None)


def test_sparse_decode_validation_order_on_host():
    good = ds.shape(1, 2, 2, 128, 100, 128, 8, 10)
    assert _sparse(good, K=None) == ds.DS_ERR_NULL
    assert _sparse(good, q=None) == ds.DS_ERR_NULL
    assert _sparse(None) == ds.DS_ERR_NULL
    assert _sparse(ds.shape(1, 2, 2, 128, 100, 128, 0, 10)) == ds.DS_ERR_SHAPE
    assert _sparse(ds.shape(1, 2, 2, 128, 100, 128, 129, 10)) == ds.DS_ERR_SHAPE
    assert _sparse(ds.shape(1, 2, 2, 128, 100, 128, 8, 0)) == ds.DS_ERR_SHAPE
    assert _sparse(ds.shape(1, 2, 2, 128, 0, 128, 8, 10)) == ds.DS_ERR_SHAPE
    assert _sparse(ds.shape(1, 3, 2, 128, 100, 128, 8, 10)) == ds.DS_ERR_SHAPE
    assert _sparse(good, K=ctypes.c_void_p(0x10010)) == ds.DS_ERR_ALIGN
    assert _sparse(good, label=ctypes.c_void_p(0x10002)) == ds.DS_ERR_ALIGN
    assert _sparse(good, ws_bytes=16) == ds.DS_ERR_WORKSPACE


@settings(max_examples=200, deadline=None)
@given(B=st.integers(-1, 3), Hq=st.integers(-1, 9), Hkv=st.integers(-1, 9), d=st.sampled_from([0, 64, 127, 128, 256]),
       L=st.integers(-5, 70000), extra=st.integers(-3, 100), r=st.integers(-2, 130), k=st.integers(-2, 70000))
def test_invalid_shapes_never_reach_the_device(B, Hq, Hkv, d, L, extra, r, k):
    """Any shape that breaks a documented rule is refused with DS_ERR_SHAPE and a
    zero workspace size; the pointers here are fake, so a launch would crash."""
    L_max = L + extra
    valid = (B >= 1 and Hq >= 1 and Hkv >= 1 and d == 128 and Hq % max(Hkv, 1) == 0 and 1 <= L <= L_max
             and 1 <= r <= d and k >= 1)
    shp = ds.shape(B, Hq, Hkv, d, L, L_max, r, k)
    if valid:
        assert ds.ds_workspace_bytes(shp) > 0
        assert _sparse(shp, ws_bytes=0) == ds.DS_ERR_WORKSPACE
    else:
        assert ds.ds_workspace_bytes(shp) == 0 or not (1 <= r <= d and k >= 1)
        assert _sparse(shp) == ds.DS_ERR_SHAPE
        lib = ds.lib()
        assert lib.ds_select(FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, ctypes.byref(shp), None) == ds.DS_ERR_SHAPE


def test_other_entry_points_refuse_null_and_bad_sizes():
    lib = ds.lib()
    good = ds.shape(1, 2, 2, 128, 100, 128, 8, 10)
    g = ctypes.byref(good)
    assert lib.ds_dense_decode(None, FAKE, FAKE, FAKE, FAKE, 1 << 40, g, None) == ds.DS_ERR_NULL
    assert lib.ds_dense_decode(FAKE, FAKE, FAKE, FAKE, FAKE, 8, g, None) == ds.DS_ERR_WORKSPACE
    assert lib.ds_build_label(FAKE, None, FAKE, g, None) == ds.DS_ERR_NULL
    assert lib.ds_build_label(ctypes.c_void_p(0x10008), FAKE, FAKE, g, None) == ds.DS_ERR_ALIGN
    assert lib.ds_append_label(FAKE, FAKE, FAKE, g, -1, 1, None) == ds.DS_ERR_SHAPE
    assert lib.ds_append_label(FAKE, FAKE, FAKE, g, 120, 9, None) == ds.DS_ERR_SHAPE
    assert lib.ds_attend_rows(FAKE, None, FAKE, FAKE, 1 << 40, g, None) == ds.DS_ERR_NULL
    assert lib.ds_gather_rows_host(FAKE, FAKE, None, FAKE, g, None) == ds.DS_ERR_NULL
    assert lib.ds_probe_stream_read(FAKE, 24, FAKE, None) == ds.DS_ERR_SHAPE
    assert lib.ds_probe_stream_read(None, 32, FAKE, None) == ds.DS_ERR_NULL
    assert lib.ds_workspace_errors(None, 1 << 20, g, None, None, None) == ds.DS_ERR_NULL
    assert lib.ds_workspace_errors(FAKE, 8, g, None, None, None) == ds.DS_ERR_WORKSPACE
    assert lib.ds_tune_set(7, 0) == ds.DS_ERR_SHAPE
    assert lib.ds_tune_set(5, 4) == ds.DS_OK and lib.ds_tune_get(5) == 4 and lib.ds_tune_set(5, 0) == ds.DS_OK
    assert lib.ds_tune_set(1, 100) == ds.DS_ERR_SHAPE
    assert lib.ds_tune_set(1, 512) == ds.DS_OK and lib.ds_tune_get(1) == 512
    assert lib.ds_tune_set(1, 0) == ds.DS_OK
    assert lib.ds_profile_kernel_count() > 5 and lib.ds_profile_kernel_name(1) == b"k_score"


@pytest.mark.parametrize("name", ["C1", "C4a"])
def test_calibrate_channels_matches_oracle_and_seeded_outliers(name):
    w = WORKLOADS[name]
    qc, kc = make_calibration_numpy(w, layer=2)
    for mode in (ds.DS_CALIB_Q, ds.DS_CALIB_K, ds.DS_CALIB_QK):
        for r in (1, 8, 16, 128):
            got = ds.ds_calibrate_channels(qc, kc, r, mode)
            assert np.array_equal(got, O.calibrate(qc, kc, r, mode)[0])
        assert np.array_equal(ds.ds_calibrate_channels(qc, kc, 8, mode), outlier_channels(w.Hkv, w.d, 2))
    with pytest.raises(ds.DsError) as e:
        ds.ds_calibrate_channels(qc, kc, 0, 2)
    assert e.value.status == ds.DS_ERR_SHAPE
    with pytest.raises(ds.DsError):
        ds.ds_calibrate_channels(qc, kc, 8, 5)


def test_calibrate_tie_rule_and_small_values():
    # subnormal and equal importances: lower channel wins, output ascending
    qc = np.zeros((3, 2, 6), np.float16); kc = np.zeros((3, 1, 6), np.float16)
    qc[..., 1] = 6e-8; qc[..., 4] = 6e-8; qc[..., 5] = 1.0
    kc[..., :] = 1.0
    assert ds.ds_calibrate_channels(qc, kc, 2, ds.DS_CALIB_Q).tolist() == [[1, 5]]
    assert ds.ds_calibrate_channels(qc, kc, 3, ds.DS_CALIB_QK).tolist() == [[1, 4, 5]]
    assert ds.ds_calibrate_channels(qc, kc, 2, ds.DS_CALIB_K).tolist() == [[0, 1]]
    assert np.array_equal(ds.ds_calibrate_channels(qc, kc, 3, 0), O.calibrate(qc, kc, 3, 0)[0])


def test_planner_follows_the_device_it_is_told_of():
    """Host only: the launch plan is derived from the device's compute-unit count, not from
    literals.  On the default device model (256 compute units) the headline shapes decode in one
    launch whose workgroups all fit at once; told of a device a quarter the size, the planner
    must not plan a launch whose workgroups wait for others that cannot be resident."""
    shapes = {"C3": ds.shape(1, 32, 32, 128, 65536, 65536, 8, 4096),
              "C4a": ds.shape(16, 64, 8, 128, 32768, 32768, 8, 2048)}
    for name, shp in shapes.items():
        ds.ds_pretend_device(256, 8, 160 << 10)
        try:
            big = ds.ds_plan_describe(shp)
            ds.ds_pretend_device(64, 8, 160 << 10)
            small = ds.ds_plan_describe(shp)
            ws_small = ds.ds_workspace_bytes(shp)
        finally:
            ds.ds_pretend_device(0, 0, 0)
        assert big["compute_units"] == 256 and small["compute_units"] == 64
        assert big["launches_planned"] == 1 and big["scores_itself"] == 1, (name, big)
        per_cu = 4 if big["heads_per_kv_head"] <= 2 else 3
        assert big["workgroups"] <= per_cu * 256, (name, big)
        # (either scoring becomes a launch of its own, or the units go in several launches of
        #  which each fits the small device at once)
        assert small["launches_planned"] >= 2, (name, small)
        assert small["scores_itself"] == 0 or small["workgroups"] <= small["launches_planned"] * per_cu * 64, (name, small)
        assert ws_small > 0
    # one workgroup per unit waits for nobody: the same plan on any device
    c1 = ds.shape(1, 32, 32, 128, 4096, 4096, 8, 256)
    ds.ds_pretend_device(16, 8, 160 << 10)
    try:
        assert ds.ds_plan_describe(c1)["launches_planned"] == 1
    finally:
        ds.ds_pretend_device(0, 0, 0)
    # the hook refuses devices that cannot exist
    for bad in ((0, 8, 160 << 10), (100, 8, 160 << 10), (64, 8, 1024)):
        with pytest.raises(ds.DsError):
            ds.ds_pretend_device(*bad)


def test_handed_over_arrays_are_never_read_with_plain_loads():
    """Host only, a grep over the attention kernels: the workspace arrays that one workgroup
    writes and another reads inside a launch (unit histograms, candidate list, per-chunk counts
    and offsets, partials) may be read only through ld_dev (device-scope loads).  A plain
    indexed read -- `x = cu[i]`, `... hu[i] + ...` -- could be served from a stale cache line.
    Allowed forms: the address taken for an atomic (`&hu[i]`), a clearing store (`hu[i] = 0`)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2408_07092_amd", "csrc")
    names = r"(?:cu|hu|cuh|a\.cand|a\.ndef|a\.offs_rw|a\.part|a\.hist|a\.coarse|po|pg|part_unit|ph|pc)"
    bad = []
    for fn in ("ds_attend.hip", "ds_attend_core.h"):
        for ln, line in enumerate(open(os.path.join(csrc, fn)), 1):
            code = line.split("//")[0]
            for m in re.finditer(r"(?<![\w.&])" + names + r"\s*\[", code):
                rest = code[m.end():]
                depth, i = 1, 0
                while i < len(rest) and depth:
                    depth += {"[": 1, "]": -1}.get(rest[i], 0)
                    i += 1
                after = rest[i:].lstrip()
                if after.startswith("=") and not after.startswith("=="):
                    continue                     # a store
                bad.append(f"{fn}:{ln}: {line.strip()}")
    assert not bad, "plain reads of in-launch hand-over arrays:\n" + "\n".join(bad)
