"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on seeded synthetic inputs.  Small/odd shapes span several tiles
and ragged tails; the benchmark configurations run at full size in the launch
configuration the bench times."""
import os

import numpy as np
import pytest
import torch

import paper_2408_07092_amd as ds
from oracle import ds_oracle as O
from tests.parity_util import (Case, check_decode_against_both_oracles, check_index_band, check_index_structure,
                               check_output, full_parity, to_dev)
from workloads import (WORKLOADS, Workload, make_calibration_numpy, make_layer_numpy, make_layer_torch,
                       outlier_channels)

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["score_tail", "cand_launch", "refine_attend", "unit_fused", "unit_fused_big",
                        "chunks_fused", "auto"],
                autouse=True)
def decode_path(request):
    """Every test runs on every implementation of ds_sparse_decode: the
    three-launch path with the exact threshold settled either in the scoring
    launch's tail or in a candidate launch of its own, scoring followed by the
    launch that refines the threshold behind the attention, that launch with one
    workgroup per unit doing the scoring as well (chunks of 6144 tokens: units up
    to that length; chunks of 16384 tokens: the variant of a workgroup that has a CU to
    itself), the same with several scoring workgroups per unit, and the library's own
    choice."""
    mode, refine, chunk, _ = {"score_tail": (1, 2, 0, 0),
                                  "cand_launch": (1, 1, 0, 0), "refine_attend": (4, 1, 0, 0), "unit_fused": (4, 0, 6144, 0),
                                  "unit_fused_big": (4, 0, 16384, 0),
                                  "chunks_fused": (4, 2, 0, 0), "auto": (0, 0, 0, 0)}[request.param]
    ds.ds_tune_set(3, mode)
    ds.ds_tune_set(4, refine)
    ds.ds_tune_set(1, chunk)
    yield request.param
    ds.ds_tune_set(3, 0)
    ds.ds_tune_set(4, 0)
    ds.ds_tune_set(1, 0)


def rand_channels(Hkv, d, r, seed, sort=True):
    rng = np.random.default_rng(seed)
    rows = [rng.permutation(d)[:r] for _ in range(Hkv)]
    return np.stack([np.sort(x) if sort else x for x in rows]).astype(np.int32)


def small_workload(B, Hq, Hkv, L, r, k):
    return Workload("t", B, Hq, Hkv, 128, L, r, k, 1)


# ---------------------------------------------------------------- odd shapes
@pytest.mark.parametrize("B,Hq,Hkv,L,L_max,r,k", [
    (1, 1, 1, 1, 1, 8, 1),            # single token
    (1, 2, 2, 5, 8, 8, 3),
    (2, 4, 4, 63, 64, 8, 7),
    (1, 3, 3, 257, 300, 16, 16),
    (2, 2, 2, 1000, 1000, 8, 62),     # ragged chunk tail
    (1, 4, 4, 4097, 4100, 8, 256),    # one token past a tile
    (1, 2, 2, 2048, 2048, 8, 2048),   # k = L
    (1, 2, 2, 300, 512, 8, 999),      # k > L clamps
    (1, 2, 2, 3000, 3000, 8, 1),      # k = 1
    (1, 2, 2, 1500, 1500, 1, 100),    # r = 1 (scalar label path)
    (1, 2, 2, 1500, 1500, 3, 100),    # odd r
    (1, 2, 2, 1500, 1500, 24, 100),   # r % 8 == 0, generic vector path
    (1, 1, 1, 700, 700, 128, 50),     # r = d
    (3, 8, 2, 900, 1024, 8, 57),      # GQA group 4
    (2, 16, 2, 777, 800, 8, 40),      # GQA group 8
    (1, 6, 2, 520, 520, 16, 33),      # GQA group 3 (no power-of-two tile)
    (1, 32, 2, 400, 400, 8, 25),      # GQA group 16 (two passes of 8)
    (1, 8, 2, 9000, 9000, 8, 500),    # GQA group 4, several chunks per unit that score themselves
    (1, 16, 2, 10000, 10016, 16, 700),  # GQA group 8, r = 16, the same
    (1, 6, 2, 9001, 9004, 8, 300),    # GQA group 3, the same with a ragged tail
    (1, 32, 2, 8200, 8200, 8, 513),   # GQA group 16, the same
    (2, 4, 4, 6000, 6000, 8, 375),    # single heads, 4K < L <= 8K with few units
])
def test_small_shapes(B, Hq, Hkv, L, L_max, r, k):
    w = small_workload(B, Hq, Hkv, L, r, k)
    t = make_layer_numpy(w, layer=L % 7, L_max=L_max)
    ch = rand_channels(Hkv, 128, r, seed=L + r, sort=(r != 3))
    case = Case(t["q"], t["K"], t["V"], ch, L, k)
    full_parity(case, what=f"B{B} Hq{Hq} Hkv{Hkv} L{L} r{r} k{k}")


def test_identity_channels_k_eq_L_is_dense():
    w = small_workload(1, 2, 2, 640, 128, 640)
    t = make_layer_numpy(w)
    ch = np.tile(np.arange(128, dtype=np.int32), (2, 1))
    case = Case(t["q"], t["K"], t["V"], ch, 640, 640)
    lab = case.gpu_build_label()
    assert np.array_equal(lab.view(np.uint16), t["K"].view(np.uint16))
    out, idx = case.gpu_sparse()
    assert (idx == np.arange(640)).all()
    check_output(out, O.dense_decode(t["q"], t["K"], t["V"], 640), "k=L vs dense oracle")
    check_output(case.gpu_dense(), O.dense_decode(t["q"], t["K"], t["V"], 640), "dense")


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        Hkv = int(rng.choice([1, 2, 3, 5]))
        G = int(rng.choice([1, 1, 2, 3, 4, 8]))
        B = int(rng.integers(1, 4))
        L = int(rng.choice([rng.integers(1, 40), rng.integers(40, 1200), rng.integers(1200, 7000), rng.integers(8200, 14000)]))
        L_max = L + int(rng.choice([0, 1, 3, 17]))
        r = int(rng.choice([1, 2, 5, 8, 8, 8, 16, 24]))
        k = int(max(1, min(L + 2, rng.choice([1, L // 16 + 1, L // 4 + 1, L]))))
        out.append((B, Hkv * G, Hkv, L, L_max, r, k))
    return out


@pytest.mark.parametrize("B,Hq,Hkv,L,L_max,r,k", _random_shapes(14, seed=314159) + _random_shapes(10, seed=2718))
def test_random_shapes(B, Hq, Hkv, L, L_max, r, k):
    """A seeded draw of shapes (head groups, ragged lengths, padded caches, r and k at
    both ends of their ranges) through every stage against the oracle."""
    w = small_workload(B, Hq, Hkv, L, r, k)
    t = make_layer_numpy(w, L_max=L_max)
    case = Case(t["q"], t["K"], t["V"], rand_channels(Hkv, 128, r, seed=L + 7 * r), L, k)
    full_parity(case, check_dense=(L < 3000), what=f"random shape {(B, Hq, Hkv, L, L_max, r, k)}")


@pytest.mark.parametrize("L,r,k", [(8192, 8, 512), (5000, 16, 300)])
def test_many_units_one_workgroup_each(L, r, k):
    """256 units of a length one workgroup takes: the library's own choice is a single
    launch per layer (fp16 labels) or scoring plus one workgroup per unit (other label
    sources); every variant of the fixture runs the same comparison."""
    w = small_workload(8, 32, 32, L, r, k)
    t = make_layer_torch(w, "cuda", layer=3)
    ch = rand_channels(32, 128, r, seed=L)
    case = Case.from_torch(t, ch, L, k)
    full_parity(case, check_dense=False, what=f"256 units x {L}")
    _q4_parity(case.q_h, case.K_h, case.V_h, ch, L, k, f"256 units x {L}, q4")


# ---------------------------------------------------------------- ties
@pytest.mark.parametrize("L,k,G", [(1200, 100, 1), (5000, 313, 1), (2500, 77, 4)])
def test_integer_scores_many_exact_ties(L, k, G):
    """Small-integer q and K make thousands of equal scores: the lowest token
    indices must win, exactly as in the oracle's full sort."""
    rng = np.random.default_rng(L)
    Hkv = 2
    q = rng.integers(-2, 3, size=(1, Hkv * G, 128)).astype(np.float16)
    K = rng.integers(-2, 3, size=(1, Hkv, L, 128)).astype(np.float16)
    V = rng.standard_normal((1, Hkv, L, 128)).astype(np.float16)
    ch = rand_channels(Hkv, 128, 8, seed=1)
    case = Case(q, K, V, ch, L, k)
    full_parity(case, check_dense=False, what="ties")


@pytest.mark.parametrize("shape", ["rising", "falling", "sawtooth"])
def test_scores_trending_along_the_sequence(shape):
    """Approximate scores that drift with the position: a chunk's own histogram then says little
    about the unit's threshold (chunks far below it select nothing, chunks far above it
    everything), whichever way a workgroup guesses before the unit's histogram is complete."""
    L, k, Hkv = 20000, 1250, 2
    rng = np.random.default_rng(7)
    ch = rand_channels(Hkv, 128, 8, seed=5)
    q = rng.standard_normal((1, Hkv, 128)).astype(np.float16)
    K = rng.standard_normal((1, Hkv, L, 128)).astype(np.float16)
    t = np.arange(L, dtype=np.float64)
    trend = {"rising": t / L, "falling": 1.0 - t / L, "sawtooth": (t % 3000) / 3000.0}[shape] * 6.0 - 3.0
    for h in range(Hkv):
        q[0, h, ch[h]] = np.float16(1.0)
        K[0, h][:, ch[h]] = (trend[:, None] + 0.25 * rng.standard_normal((L, 8))).astype(np.float16)
    V = rng.standard_normal((1, Hkv, L, 128)).astype(np.float16)
    case = Case(q, K, V, ch, L, k)
    full_parity(case, check_dense=False, what="trend " + shape)


def test_all_scores_equal_selects_first_k_tokens():
    L, k = 3000, 129
    q = np.zeros((1, 2, 128), np.float16)                  # every approximate score is +0
    rng = np.random.default_rng(0)
    K = rng.standard_normal((1, 2, L, 128)).astype(np.float16)
    K[0, 1] = -np.abs(K[0, 1])                             # and -0 * x products stay zero
    V = rng.standard_normal((1, 2, L, 128)).astype(np.float16)
    case = Case(q, K, V, rand_channels(2, 128, 8, 3), L, k)
    case.gpu_build_label()
    out, idx = case.gpu_sparse()
    assert (idx == np.arange(k)).all()
    full_parity(case, check_dense=False, what="all equal")


def test_negative_zero_ties_with_positive_zero():
    L, k = 600, 10
    q = np.zeros((1, 1, 128), np.float16); q[0, 0, 5] = -1.0
    K = np.zeros((1, 1, L, 128), np.float16)               # scores are -1 * (+0) = -0 and -1 * (-0) = +0
    K[0, 0, ::2, 5] = -0.0
    K[0, 0, 300:, 5] = 1.0                                 # clearly lower scores (-1)
    V = np.random.default_rng(1).standard_normal((1, 1, L, 128)).astype(np.float16)
    ch = np.array([[5, 6, 7, 8, 9, 10, 11, 12]], np.int32)
    case = Case(q, K, V, ch, L, k)
    case.gpu_build_label()
    _, idx = case.gpu_sparse()
    assert idx[0, 0].tolist() == list(range(10))
    full_parity(case, check_dense=False, what="signed zeros")


def test_a_few_hundred_tied_candidates_are_ranked_by_token(decode_path):
    """Up to 256 keys in the threshold bin take the direct ranking (one candidate per thread): with
    200 equal scores at the threshold and room for 37 of them, the 37 lowest tokens must win; with
    two distinct scores inside one bin, the higher one first."""
    L, k = 3000, 37
    q = np.zeros((1, 1, 128), np.float16); q[0, 0, 5] = 1.0
    K = np.zeros((1, 1, L, 128), np.float16)
    K[0, 0, :, 5] = -1.0
    tied = np.arange(100, 2100, 10)                          # 200 tokens, spread over the chunks
    K[0, 0, tied, 5] = 1.0
    V = np.random.default_rng(3).standard_normal((1, 1, L, 128)).astype(np.float16)
    ch = np.array([[5, 6, 7, 8, 9, 10, 11, 12]], np.int32)
    case = Case(q, K, V, ch, L, k)
    case.gpu_build_label()
    _, idx = case.gpu_sparse()
    assert idx[0, 0].tolist() == tied[:37].tolist()
    full_parity(case, check_dense=False, what="200 ties")
    K[0, 0, tied[50:90], 5] = 1.0009765625                   # same bin (the next binary16), 40 higher keys
    case = Case(q, K, V, ch, L, 60)
    case.gpu_build_label()
    _, idx = case.gpu_sparse()
    assert idx[0, 0].tolist() == sorted(tied[50:90].tolist() + tied[:20].tolist())
    full_parity(case, check_dense=False, what="two keys in one bin")


# ---------------------------------------------------------------- label cache
def test_append_label_equals_build_and_error_codes():
    w = small_workload(2, 4, 4, 500, 8, 10)
    t = make_layer_numpy(w, L_max=512)
    ch = rand_channels(4, 128, 8, 9)
    case = Case(t["q"], t["K"], t["V"], ch, 500, 10)
    full = case.gpu_build_label().copy()
    case.label.zero_()
    shp = ds.shape(2, 4, 4, 128, 490, 512, 8, 10)
    ds.ds_build_label(case.K, case.ch, case.label, shp)
    ds.ds_append_label(case.K, case.ch, case.label, shp, 490, 1)      # one decode step
    ds.ds_append_label(case.K, case.ch, case.label, shp, 491, 9)      # a burst
    ds.ds_append_label(case.K, case.ch, case.label, shp, 500, 0)      # nothing
    torch.cuda.synchronize()
    assert np.array_equal(case.label.cpu().numpy().view(np.uint16), full.view(np.uint16))
    with pytest.raises(ds.DsError) as e:
        ds.ds_append_label(case.K, case.ch, case.label, shp, 510, 3)
    assert e.value.status == ds.DS_ERR_SHAPE


def test_device_entry_points_reject_bad_arguments_without_touching_outputs():
    w = small_workload(1, 2, 2, 300, 8, 16)
    t = make_layer_numpy(w)
    case = Case(t["q"], t["K"], t["V"], rand_channels(2, 128, 8, 4), 300, 16)
    case.gpu_build_label()
    out = torch.full((1, 2, 128), 5.0, dtype=torch.float32, device="cuda")
    small_ws = torch.empty(64, dtype=torch.uint8, device="cuda")
    cases = [
        (lambda: ds.ds_sparse_decode(case.q, case.label, case.K, case.V, case.ch, out, None, small_ws, case.shape),
         ds.DS_ERR_WORKSPACE),
        (lambda: ds.ds_sparse_decode(case.q, case.label, None, case.V, case.ch, out, None, case.ws, case.shape),
         ds.DS_ERR_NULL),
        (lambda: ds.ds_sparse_decode(case.q, case.label, case.K, case.V, case.ch, out, None, case.ws,
                                     ds.shape(1, 2, 2, 64, 300, 300, 8, 16)), ds.DS_ERR_SHAPE),
        (lambda: ds.ds_sparse_decode(case.q, case.label, case.K, case.V, case.ch, out, None, case.ws,
                                     ds.shape(1, 2, 2, 128, 301, 300, 8, 16)), ds.DS_ERR_SHAPE),
        (lambda: ds.ds_sparse_decode(case.q, case.label, case.K.view(-1)[8:].view(-1), case.V, case.ch, out, None,
                                     case.ws, case.shape), ds.DS_ERR_ALIGN),
        (lambda: ds.ds_dense_decode(case.q, case.K, case.V, out, small_ws, case.shape), ds.DS_ERR_WORKSPACE),
        (lambda: ds.ds_select(case.q, case.label, case.ch, None, case.ws, case.shape), ds.DS_ERR_NULL),
    ]
    for fn, want in cases:
        with pytest.raises(ds.DsError) as e:
            fn()
        assert e.value.status == want
    torch.cuda.synchronize()
    assert (out == 5.0).all()


# ---------------------------------------------------------------- offload split path
def test_select_gather_from_pinned_host_attend_rows():
    w = small_workload(1, 4, 4, 3000, 8, 200)
    t = make_layer_numpy(w)
    ch = rand_channels(4, 128, 8, 12)
    case = Case(t["q"], t["K"], t["V"], ch, 3000, 200)
    lab_ref = case.oracle_label()
    case.gpu_build_label()
    Kp = torch.from_numpy(t["K"]).pin_memory()
    Vp = torch.from_numpy(t["V"]).pin_memory()
    idx = torch.full((1, 4, 200), -7, dtype=torch.int32, device="cuda")
    rows = torch.empty((1, 4, 200, 2, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((1, 4, 128), dtype=torch.float32, device="cuda")
    ds.ds_select(case.q, case.label, case.ch, idx, case.ws, case.shape)
    ds.ds_gather_rows_host(Kp, Vp, idx, rows, case.shape)
    ds.ds_attend_rows(case.q, rows, out, case.ws, case.shape)
    torch.cuda.synchronize()
    idx_h, rows_h = idx.cpu().numpy(), rows.cpu().numpy()
    check_decode_against_both_oracles(idx_h, out.cpu().numpy(), t["q"], lab_ref, t["K"], t["V"], ch, 3000, 200,
                                      "offload split path")
    for h in range(4):
        assert np.array_equal(rows_h[0, h, :, 0].view(np.uint16), t["K"][0, h, idx_h[0, h]].view(np.uint16))
        assert np.array_equal(rows_h[0, h, :, 1].view(np.uint16), t["V"][0, h, idx_h[0, h]].view(np.uint16))


def test_offload_pipeline_double_buffer_matches_oracle_over_layers():
    """Five layers through the two-slot pipeline (select / host-row fetch / attend on
    three streams), twice, against the oracle per layer."""
    from paper_2408_07092_amd.offload import OffloadDecoder
    w = small_workload(2, 4, 2, 2500, 8, 150)          # GQA group 2, ragged L
    shp = ds.shape(w.B, w.Hq, w.Hkv, w.d, w.L, w.L, w.r, w.k)
    layers, outs, refs = [], [], []
    for l in range(5):
        t = make_layer_numpy(w, layer=l)
        ch = rand_channels(w.Hkv, 128, 8, 100 + l)
        lab_ref = O.build_label(t["K"], ch, w.L)
        # the pipeline hands back outputs only: the reference is the float64 definition, on the
        # binary32-order selection (which the band check ties to the float64 one) where they differ
        _, idx32 = O.sparse_decode(t["q"], lab_ref, t["K"], t["V"], ch, w.L, w.k, precision=32)
        out64, _, sc64, srt64 = O.sparse_decode(t["q"], lab_ref, t["K"], t["V"], ch, w.L, w.k, precision=64,
                                                want_scores=True)
        differing = check_index_band(idx32, sc64, srt64, w.L, w.k)
        refs.append(out64 if differing == 0 else O.attend_idx(t["q"], t["K"], t["V"], idx32))
        layers.append((to_dev(t["q"]), to_dev(lab_ref), to_dev(ch),
                       torch.from_numpy(t["K"]).pin_memory(), torch.from_numpy(t["V"]).pin_memory()))
        outs.append(torch.zeros((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda"))
    dec = OffloadDecoder(shp)
    first = None
    for rep in range(2):
        dec.decode(layers, outs)
        torch.cuda.synchronize()
        got = [o.cpu().numpy() for o in outs]
        for l in range(5):
            check_output(got[l], refs[l], f"offload pipeline layer {l}")
        blob = b"".join(g.tobytes() for g in got)
        first = first or blob
        assert blob == first


# ---------------------------------------------------------------- calibration feeds the path
def test_calibrated_channels_drive_selection_c1():
    w = WORKLOADS["C1"]
    qc, kc = make_calibration_numpy(w)
    ch = ds.ds_calibrate_channels(qc, kc, w.r, ds.DS_CALIB_QK)
    assert np.array_equal(ch, outlier_channels(w.Hkv, w.d))
    assert np.array_equal(ch, O.calibrate(qc, kc, w.r, 2)[0])
    t = make_layer_numpy(w)
    case = Case(t["q"], t["K"], t["V"], ch, w.L, w.k)
    rep = full_parity(case, what="C1")
    print("C1", rep)


# ---------------------------------------------------------------- full-size configurations
def _full_config(name, check_dense_heads=None):
    w = WORKLOADS[name]
    qc, kc = make_calibration_numpy(w)
    mode = ds.DS_CALIB_QK if w.G == 1 else ds.DS_CALIB_Q
    ch = ds.ds_calibrate_channels(qc, kc, w.r, mode)
    t = make_layer_torch(w, "cuda", layer=0)
    case = Case.from_torch(t, ch, w.L, w.k)
    rep = full_parity(case, check_dense=False, what=name)
    # dense: compare a sample of batches (the oracle's dense pass is the slow part)
    nb = min(w.B, 2)
    d_gpu = case.gpu_dense()
    d_ref = O.dense_decode(case.q_h[:nb], case.K_h[:nb], case.V_h[:nb], w.L)
    rep["dense"] = check_output(d_gpu[:nb], d_ref, name + " dense")
    print(name, rep)


def _decode_launches(case):
    """Kernel name -> launches of one ds_sparse_decode call without an index list."""
    case.gpu_sparse(want_idx=False)
    ds.ds_profile_enable(True)
    ds.ds_profile_reset()
    case.gpu_sparse(want_idx=False)
    torch.cuda.synchronize()
    rep = {k: n for k, (ms, n) in ds.ds_profile_read().items() if n}
    ds.ds_profile_enable(False)
    return rep


@pytest.mark.parametrize("name", ["C2", "C3", "C4a", "C4b"])
def test_full_configs_decode_in_one_launch_by_default(name, decode_path):
    """The benchmark configurations take the path the bench times: scoring, selection and
    attention in a single launch per layer (the parity of that path is checked by the full-size
    tests below under the same default)."""
    if decode_path != "auto":
        pytest.skip("default launch shape only")
    w = WORKLOADS[name]
    t = make_layer_torch(w, "cuda", layer=0)
    ch = outlier_channels(w.Hkv, w.d) if w.r == 8 else np.tile(np.arange(w.r, dtype=np.int32), (w.Hkv, 1))
    case = Case.from_torch(t, ch, w.L, w.k)
    case.gpu_build_label()
    assert _decode_launches(case) == {"k_refine_attend": 1}


def test_many_single_head_units_of_32k_tokens_decode_in_one_launch(decode_path):
    """128 single-head units of 32K tokens: four workgroups per unit with chunks of 8192 tokens is
    what the device holds at once (LDS), so that scoring, selection and attention stay one launch;
    parity of that launch at full size against the oracle."""
    if decode_path != "auto":
        pytest.skip("default launch shape only")
    w = Workload("long_single_heads", 4, 32, 32, 128, 32768, 8, 2048, 1)
    t = make_layer_torch(w, "cuda", layer=1)
    case = Case.from_torch(t, outlier_channels(w.Hkv, w.d), w.L, w.k)
    rep = full_parity(case, check_dense=False, what="128 units x 32K")
    plan = ds.ds_plan_describe(case.shape, 0)
    assert plan["workgroups_per_unit"] == 4 and plan["tokens_per_workgroup"] == 8192, plan
    assert _decode_launches(case) == {"k_refine_attend": 1}
    print("128 units x 32K", rep)


def test_full_config_c2():
    _full_config("C2")


def test_full_config_c3_headline():
    _full_config("C3")


def test_full_config_c4a_gqa8():
    _full_config("C4a")


def test_full_config_c4b_gqa4():
    _full_config("C4b")


def test_full_config_c5_offload_rows_from_pinned_host():
    """L = 256K, K/V in pinned host memory, label cache on the device: select on
    the GPU, fetch the k rows over the host link, attend over them."""
    w = WORKLOADS["C5"]
    qc, kc = make_calibration_numpy(w)
    ch = ds.ds_calibrate_channels(qc, kc, w.r, ds.DS_CALIB_QK)
    t = make_layer_torch(w, "cuda", layer=0, pin_kv=True)
    Kp, Vp = t["K"], t["V"]
    K_h, V_h, q_h = Kp.numpy(), Vp.numpy(), t["q"].cpu().numpy()
    shp = ds.shape(w.B, w.Hq, w.Hkv, w.d, w.L, w.L, w.r, w.k)
    # the label cache is built from a temporary device copy of K; K then leaves the device
    label = torch.empty((w.B, w.Hkv, w.L, w.r), dtype=torch.float16, device="cuda")
    ch_d = to_dev(ch)
    Kd = Kp.cuda()
    ds.ds_build_label(Kd, ch_d, label, shp)
    torch.cuda.synchronize()
    del Kd
    torch.cuda.synchronize()
    lab_ref = O.build_label(K_h, ch, w.L)
    assert np.array_equal(label.cpu().numpy().view(np.uint16), lab_ref.view(np.uint16))
    ws = ds.ds_workspace_alloc(shp)
    idx = torch.empty((w.B, w.Hkv, w.k), dtype=torch.int32, device="cuda")
    rows = torch.empty((w.B, w.Hkv, w.k, 2, w.d), dtype=torch.float16, device="cuda")
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
    ds.ds_select(t["q"], label, ch_d, idx, ws, shp)
    ds.ds_gather_rows_host(Kp, Vp, idx, rows, shp)
    ds.ds_attend_rows(t["q"], rows, out, ws, shp)
    torch.cuda.synchronize()
    print("C5", check_decode_against_both_oracles(idx.cpu().numpy(), out.cpu().numpy(), q_h, lab_ref, K_h, V_h, ch,
                                                  w.L, w.k, "C5 offload"))


def test_nolabel_rejects_bad_arguments_and_matches_label_path_bytes():
    w = WORKLOADS["C1"]
    t = make_layer_numpy(w)
    case = Case(t["q"], t["K"], t["V"], outlier_channels(w.Hkv, w.d), w.L, w.k)
    case.gpu_build_label()
    out_l, idx_l = case.gpu_sparse()
    out_n, idx_n = case.gpu_sparse_nolabel()
    assert np.array_equal(idx_l, idx_n)
    # the co-resident launches order their partial sums differently, and so does the variant of
    # a workgroup that has a CU to itself (rows reach the slots in another order)
    if ds.ds_tune_get(3) not in (2, 3) and ds.ds_tune_get(1) <= 8192:
        assert out_l.tobytes() == out_n.tobytes()
    else:
        assert np.allclose(out_l, out_n, rtol=1e-4, atol=1e-5)
    out = torch.zeros((case.B, case.Hq, case.d), dtype=torch.float32, device="cuda")
    with pytest.raises(ds.DsError) as e:
        ds.ds_sparse_decode_nolabel(case.q, None, case.V, case.ch, out, None, case.ws, case.shape)
    assert e.value.status == ds.DS_ERR_NULL
    bad = ds.shape(case.B, case.Hq, case.Hkv, case.d, case.L_max + 1, case.L_max, case.r, case.k)
    with pytest.raises(ds.DsError) as e:
        ds.ds_sparse_decode_nolabel(case.q, case.K, case.V, case.ch, out, None, case.ws, bad)
    assert e.value.status == ds.DS_ERR_SHAPE
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0


# ---------------------------------------------------------------- interleaved K|V cache, fused append
@pytest.mark.parametrize("B,Hq,Hkv,L,L_max,r,k", [
    (2, 4, 4, 777, 800, 8, 50),
    (1, 16, 2, 3000, 3072, 16, 200),     # GQA 8 on the matrix cores
    (1, 2, 2, 9000, 9000, 8, 600),       # long enough for the refine-and-attend launch
])
def test_interleaved_cache_append_and_decode(B, Hq, Hkv, L, L_max, r, k):
    """Prefill L - 5 tokens, append 3 + 2 with the fused append (both layouts),
    decode over the interleaved cache: caches and label bit-exact against the
    oracle's append, decode against the oracle on the separate K and V."""
    rng = np.random.default_rng(L)
    w = small_workload(B, Hq, Hkv, L, r, k)
    t = make_layer_numpy(w, L_max=L_max)
    q, K, V = t["q"], t["K"], t["V"]
    ch = rand_channels(Hkv, 128, r, seed=L)
    L0 = L - 5
    # oracle: caches holding L0 tokens, then two appends
    K_o, V_o = K.copy(), V.copy()
    K_o[:, :, L0:] = 0; V_o[:, :, L0:] = 0
    lab_o = O.build_label(K_o, ch, L0)
    steps = [(L0, 3), (L0 + 3, 2)]
    for t0, n in steps:
        O.append_kv(K[:, :, t0:t0 + n].copy(), V[:, :, t0:t0 + n].copy(), K_o, V_o, ch, lab_o, t0)
    # HIP path, separate layout
    shp = ds.shape(B, Hq, Hkv, 128, L, L_max, r, k)
    shp0 = ds.shape(B, Hq, Hkv, 128, L0, L_max, r, k)
    K_d, V_d = to_dev(K_o * 0), to_dev(V_o * 0)
    K_d[:, :, :L0] = to_dev(K[:, :, :L0]); V_d[:, :, :L0] = to_dev(V[:, :, :L0])
    ch_d = to_dev(ch)
    lab_d = torch.zeros((B, Hkv, L_max, r), dtype=torch.float16, device="cuda")
    ds.ds_build_label(K_d, ch_d, lab_d, shp0)
    # HIP path, interleaved layout
    KV_d = torch.zeros((B, Hkv, L_max, 2, 128), dtype=torch.float16, device="cuda")
    KV_d[:, :, :L0, 0] = K_d[:, :, :L0]; KV_d[:, :, :L0, 1] = V_d[:, :, :L0]
    lab_i = torch.zeros_like(lab_d)
    ds.ds_build_label_kv(KV_d, ch_d, lab_i, shp0)
    for t0, n in steps:
        kn, vn = to_dev(K[:, :, t0:t0 + n]), to_dev(V[:, :, t0:t0 + n])
        ds.ds_append_kv(kn, vn, K_d, V_d, ch_d, lab_d, shp, t0, n, ds.DS_KV_SPLIT)
        ds.ds_append_kv(kn, vn, KV_d, None, ch_d, lab_i, shp, t0, n, ds.DS_KV_INTERLEAVED)
    torch.cuda.synchronize()
    for got, want in ((K_d, K_o), (V_d, V_o), (lab_d, lab_o), (lab_i, lab_o),
                      (KV_d, O.interleave_kv(K_o, V_o))):
        assert np.array_equal(got.cpu().numpy().view(np.uint16), want.view(np.uint16))
    # decode over the interleaved cache
    ws = ds.ds_workspace_alloc(shp)
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((B, Hkv, k), -7, dtype=torch.int32, device="cuda")
    ds.ds_sparse_decode_kv(to_dev(q), lab_i, KV_d, ch_d, out, idx, ws, shp)
    torch.cuda.synchronize()
    check_decode_against_both_oracles(idx.cpu().numpy(), out.cpu().numpy(), q, lab_o, K_o, V_o, ch, L, k,
                                      "interleaved decode")
    # bad layout / range are refused before anything is enqueued
    with pytest.raises(ds.DsError) as e:
        ds.ds_append_kv(to_dev(K[:, :, :2]), to_dev(V[:, :, :2]), K_d, V_d, ch_d, lab_d, shp, L_max - 1, 2)
    assert e.value.status == ds.DS_ERR_SHAPE
    with pytest.raises(ds.DsError) as e:
        ds.ds_append_kv(to_dev(K[:, :, :2]), to_dev(V[:, :, :2]), K_d, None, ch_d, lab_d, shp, 0, 2, ds.DS_KV_SPLIT)
    assert e.value.status == ds.DS_ERR_NULL


# ---------------------------------------------------------------- query prediction + offload schedule
@pytest.mark.parametrize("B,Dm,N", [(1, 8, 1), (1, 4096, 4096), (3, 520, 77), (4, 1024, 256), (9, 2048, 128),
                                    (2, 8192, 64)])
def test_predict_query_matches_oracle(B, Dm, N):
    """fp32 accumulation against the float64 oracle, both rounded once to fp16: equal up to
    one fp16 step of the result plus the binary32 accumulation error of the Dm products."""
    rng = np.random.default_rng(Dm + N)
    x = rng.standard_normal((B, Dm)).astype(np.float16)
    Wq = (rng.standard_normal((N, Dm)) / np.sqrt(Dm)).astype(np.float16)
    q = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    ds.ds_predict_query(to_dev(x), to_dev(Wq), q)
    torch.cuda.synchronize()
    got = q.cpu().numpy().astype(np.float64)
    ref = O.predict_query(x, Wq).astype(np.float64)
    mag = np.abs(x.astype(np.float64)) @ np.abs(Wq.astype(np.float64)).T
    tol = 2.0 ** -10 * np.abs(ref) + Dm * 2.0 ** -24 * mag + 2.0 ** -24
    assert np.isfinite(got).all() and (np.abs(got - ref) <= tol).all()
    q2 = torch.empty_like(q)
    ds.ds_predict_query(to_dev(x), to_dev(Wq), q2)
    torch.cuda.synchronize()
    assert q2.cpu().numpy().tobytes() == q.cpu().numpy().tobytes()
    with pytest.raises(ds.DsError) as e:
        ds.ds_predict_query(to_dev(x[:, :Dm - 1].copy()) if Dm > 8 else to_dev(x[:, :4].copy()),
                            to_dev(Wq[:, :Dm - 1].copy()) if Dm > 8 else to_dev(Wq[:, :4].copy()), q)
    assert e.value.status == ds.DS_ERR_SHAPE


def test_offload_schedule_with_predicted_queries_matches_oracle_over_layers():
    """Sec. 5.1 schedule: layer l's rows are selected with the query predicted from the
    previous layer's embedding (W_q of layer l applied to it), fetched from pinned host
    memory into the double buffer, and attended with the layer's real query."""
    from paper_2408_07092_amd.offload import OffloadDecoder
    B, Hq, Hkv, L, r, k, n_layers, Dm = 2, 4, 4, 3000, 8, 200, 5, 512
    w = small_workload(B, Hq, Hkv, L, r, k)
    shp = ds.shape(B, Hq, Hkv, 128, L, L, r, k)
    rng = np.random.default_rng(11)
    layers, outs, predict, host = [], [], [], []
    x_prev = rng.standard_normal((B, Dm)).astype(np.float16)
    for l in range(n_layers):
        t = make_layer_numpy(w, layer=l)
        ch = rand_channels(Hkv, 128, r, seed=l)
        Wq = (rng.standard_normal((Hq * 128, Dm)) / np.sqrt(Dm) * 4).astype(np.float16)
        Kp = torch.from_numpy(t["K"]).pin_memory()
        Vp = torch.from_numpy(t["V"]).pin_memory()
        label = torch.empty((B, Hkv, L, r), dtype=torch.float16, device="cuda")
        Kd = to_dev(t["K"])
        ds.ds_build_label(Kd, to_dev(ch), label, shp)
        torch.cuda.synchronize()
        del Kd
        q_pred = torch.zeros((B, Hq, 128), dtype=torch.float16, device="cuda")
        layers.append((to_dev(t["q"]), label, to_dev(ch), Kp, Vp))
        predict.append((to_dev(x_prev), to_dev(Wq), q_pred))
        outs.append(torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda"))
        host.append((t, ch, Wq, x_prev))
        x_prev = (x_prev.astype(np.float32) * 0.9 + 0.1 * rng.standard_normal((B, Dm))).astype(np.float16)
    dec = OffloadDecoder(shp)
    torch.cuda.synchronize()
    for rep in range(2):
        dec.decode(layers, outs, predict)
        torch.cuda.synchronize()
        for l in range(n_layers):
            t, ch, Wq, x = host[l]
            qp = predict[l][2].cpu().numpy()
            ref_q = O.predict_query(x, Wq).reshape(B, Hq, 128).astype(np.float64)
            assert np.abs(qp.astype(np.float64) - ref_q).max() <= 2.0 ** -9 * max(1.0, np.abs(ref_q).max())
            # selection with the library's approximate query, attention with the real one
            lab = O.build_label(t["K"], ch, L)
            sc = O.scores(qp, lab, ch, L, precision=32)
            idx = np.stack([[O.topk(sc[b, h], k)[0] for h in range(Hkv)] for b in range(B)]).astype(np.int32)
            ref = O.attend_idx(t["q"], t["K"], t["V"], idx)
            check_output(outs[l].cpu().numpy(), ref, f"offload+predict layer {l} rep {rep}")


# ---------------------------------------------------------------- 4-bit label cache
def _q4_parity(q, K, V, ch, L, k, what, split=None):
    """Codes and amax bit-exact against the oracle's quantiser; selection identical to the
    oracle scoring the same codes in binary32 order, inside the near-tie band of its
    float64 scores; output to the usual bar."""
    B, Hq, _ = q.shape
    _, Hkv, L_max, _ = K.shape
    r = ch.shape[1]
    W = (r + 7) // 8
    shp = ds.shape(B, Hq, Hkv, 128, L, L_max, r, k)
    K_d, V_d, q_d, ch_d = to_dev(K), to_dev(V), to_dev(q), to_dev(ch)
    codes = torch.zeros((B, Hkv, L_max, W), dtype=torch.int32, device="cuda")
    amax = torch.full((B, Hkv, r), -1.0, dtype=torch.float32, device="cuda")
    codes_ref, amax_ref = O.build_label_q4(K, ch, L)
    if split is None:
        ds.ds_build_label_q4(K_d, ch_d, codes, amax, shp)
    else:   # prefill `split` tokens' worth of amax over all L, then code in two pieces
        ds.ds_build_label_q4(K_d, ch_d, codes, amax, shp)
        codes.zero_()
        ds.ds_append_label_q4(K_d, ch_d, codes, amax, shp, 0, split)
        ds.ds_append_label_q4(K_d, ch_d, codes, amax, shp, split, L - split)
    torch.cuda.synchronize()
    assert np.array_equal(amax.cpu().numpy(), amax_ref), f"{what}: amax differs"
    assert np.array_equal(codes.cpu().numpy().view(np.uint32), codes_ref), f"{what}: 4-bit codes differ"
    ws = ds.ds_workspace_alloc(shp)
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((B, Hkv, k), -7, dtype=torch.int32, device="cuda")
    ds.ds_sparse_decode_q4(q_d, codes, amax, K_d, V_d, ch_d, out, idx, ws, shp)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    check_index_structure(idx_h, L, k)
    out32, idx32 = O.sparse_decode_q4(q, codes_ref, amax_ref, K, V, ch, L, k, precision=32)
    assert np.array_equal(idx_h, idx32), f"{what}: index sets differ from the binary32-order oracle"
    out64, idx64, sc64, srt64 = O.sparse_decode_q4(q, codes_ref, amax_ref, K, V, ch, L, k, want_scores=True)
    differing = check_index_band(idx_h, sc64, srt64, L, k)
    ref = out64 if differing == 0 else O.attend_idx(q, K, V, idx_h)
    rep = check_output(out.cpu().numpy(), ref, what)
    out2 = torch.empty_like(out)
    ds.ds_sparse_decode_q4(q_d, codes, amax, K_d, V_d, ch_d, out2, None, ws, shp)
    torch.cuda.synchronize()
    assert out2.cpu().numpy().tobytes() == out.cpu().numpy().tobytes()
    return rep


@pytest.mark.parametrize("B,Hq,Hkv,L,L_max,r,k", [
    (1, 1, 1, 1, 1, 8, 1),
    (2, 4, 4, 63, 64, 8, 7),
    (1, 3, 3, 257, 300, 16, 16),      # L_max not a multiple of 4: per-token loads
    (2, 2, 2, 1000, 1000, 8, 62),
    (1, 4, 4, 4097, 4100, 8, 256),
    (1, 2, 2, 1500, 1500, 3, 100),    # r < 8: zero nibbles
    (1, 2, 2, 1500, 1500, 11, 100),   # two words per token, second partly used
    (3, 8, 2, 900, 1024, 8, 57),      # GQA group 4
    (1, 2, 2, 9000, 9000, 8, 600),    # refine-and-attend launch
    (1, 2, 2, 9001, 9002, 11, 600),   # the same, two words per token (L_max even)
    (1, 2, 2, 9001, 9003, 8, 600),    # the same, rows that 16-byte loads cannot take: separate scoring launch
    (1, 8, 2, 9000, 9000, 8, 500),    # GQA group 4, several chunks per unit
    (1, 16, 2, 10000, 10016, 16, 700),  # GQA group 8, two words per token
])
def test_q4_label_cache_small_shapes(B, Hq, Hkv, L, L_max, r, k):
    w = small_workload(B, Hq, Hkv, L, r, k)
    t = make_layer_numpy(w, L_max=L_max)
    _q4_parity(t["q"], t["K"], t["V"], rand_channels(Hkv, 128, r, seed=L + r), L, k, "q4 small",
               split=None if L < 10 else L // 3)


def test_q4_label_cache_zero_channel_and_ties():
    """A label channel that is zero everywhere (amax = 0) and small-integer keys (many ties)."""
    rng = np.random.default_rng(5)
    L, k = 2000, 150
    q = rng.integers(-2, 3, size=(1, 2, 128)).astype(np.float16)
    K = rng.integers(-2, 3, size=(1, 2, L, 128)).astype(np.float16)
    V = rng.standard_normal((1, 2, L, 128)).astype(np.float16)
    ch = rand_channels(2, 128, 8, seed=2)
    K[0, 0, :, ch[0, 3]] = 0
    _q4_parity(q, K, V, ch, L, k, "q4 ties")


@pytest.mark.parametrize("name", ["C1", "C3", "C2"])
def test_q4_label_cache_full_config(name):
    w = WORKLOADS[name]
    qc, kc = make_calibration_numpy(w)
    ch = ds.ds_calibrate_channels(qc, kc, w.r, ds.DS_CALIB_QK)
    t = make_layer_torch(w, "cuda", layer=0)
    q, K, V = (t[x].cpu().numpy() for x in ("q", "K", "V"))
    del t
    torch.cuda.empty_cache()
    print(name, "q4", _q4_parity(q, K, V, ch, w.L, w.k, name + " q4"))


# ---------------------------------------------------------------- bounded waits that give up
@pytest.mark.parametrize("want_idx", [True, False])
def test_waits_that_give_up_end_the_launch_and_are_reported(decode_path, want_idx):
    """With a poll limit of one, workgroups stop waiting for each other at once: the launch still
    ends, the units concerned raise their error words (the result is then not to be trusted), and
    after clearing the workspace the same call is right again."""
    if decode_path not in ("auto", "chunks_fused", "refine_attend"):
        pytest.skip("launch shape 4 only")
    L, k, Hkv = 40000, 2500, 4
    rng = np.random.default_rng(11)
    q = rng.standard_normal((1, Hkv, 128)).astype(np.float16)
    K = rng.standard_normal((1, Hkv, L, 128)).astype(np.float16)
    V = rng.standard_normal((1, Hkv, L, 128)).astype(np.float16)
    case = Case(q, K, V, rand_channels(Hkv, 128, 8, seed=2), L, k)
    case.gpu_build_label()
    # (without an index list the unit's last workgroup waits for the candidate list instead of
    #  every workgroup for the exact threshold)
    good, idx = case.gpu_sparse(want_idx=want_idx)
    assert ds.ds_workspace_errors(case.ws, case.shape) == (0, 0)
    ds.ds_tune_set(5, 1)
    try:
        bad, _ = case.gpu_sparse(want_idx=want_idx)             # must return
        n_failed, code = ds.ds_workspace_errors(case.ws, case.shape)
    finally:
        ds.ds_tune_set(5, 0)
    # (workgroups that score themselves wait for their unit's histogram: the first to arrive
    #  cannot find it complete; after a separate scoring launch only the exact threshold is
    #  waited for, which may well be there in time)
    assert n_failed <= Hkv and code in (0, 6, 7, 9)
    if decode_path != "refine_attend":
        assert n_failed > 0
    # a unit whose wait ran out is all NaN, never a wrong number; the others are right
    nan_units = np.isnan(bad).all(axis=-1)[0]
    assert int(nan_units.sum()) == n_failed
    assert not np.isnan(bad[0][~nan_units]).any()
    assert bad[0][~nan_units].tobytes() == good[0][~nan_units].tobytes()
    # the error words stay up: the next call on the workspace gives NaN for those units again
    if n_failed:
        bad2, _ = case.gpu_sparse(want_idx=want_idx)
        assert (np.isnan(bad2).all(axis=-1)[0] == nan_units).all()
        assert ds.ds_workspace_errors(case.ws, case.shape)[0] == n_failed
    ds.ds_workspace_init(case.ws)
    again, idx2 = case.gpu_sparse(want_idx=want_idx)
    assert ds.ds_workspace_errors(case.ws, case.shape) == (0, 0)
    assert again.tobytes() == good.tobytes() and (not want_idx or np.array_equal(idx, idx2))


def test_grid_that_is_not_resident_takes_more_launches(decode_path):
    """The planner is told of a device a quarter the size: the one-launch shape, whose workgroups
    wait for each other, no longer fits at once, and the call must take launch shapes that need
    less room -- and give the same bytes as on the real device."""
    if decode_path != "auto":
        pytest.skip("default launch shape only")
    L, k, Hkv = 40000, 2500, 8
    rng = np.random.default_rng(12)
    q = rng.standard_normal((2, Hkv, 128)).astype(np.float16)
    K = rng.standard_normal((2, Hkv, L, 128)).astype(np.float16)
    V = rng.standard_normal((2, Hkv, L, 128)).astype(np.float16)
    case = Case(q, K, V, rand_channels(Hkv, 128, 8, seed=3), L, k)
    case.gpu_build_label()
    good, idx = case.gpu_sparse()
    plan_real = ds.ds_plan_describe(case.shape, 2)
    ds.ds_profile_reset(); ds.ds_profile_enable(True)
    try:
        ds.ds_pretend_device(8, 8, 160 << 10)      # 8 compute units: 640 workgroups cannot be resident
        plan_small = ds.ds_plan_describe(case.shape, 2)
        case.ws = ds.ds_workspace_alloc(case.shape)
        small, idx_s = case.gpu_sparse()
        launched = ds.ds_profile_read()
    finally:
        ds.ds_pretend_device(0, 0, 0)
        ds.ds_profile_enable(False); ds.ds_profile_reset()
    assert plan_real["launches"] == 1 and plan_small["launches"] > 1, (plan_real, plan_small)
    assert "k_score" in launched, launched
    assert ds.ds_workspace_errors(case.ws, case.shape) == (0, 0)
    assert np.array_equal(idx_s, idx)
    check_output(small, good.astype(np.float64), "pretended small device")


# ---------------------------------------------------------------- determinism across processes
@pytest.mark.parametrize("name", ["C1", "long", "C3", "C4a"])
def test_second_process_gives_identical_bytes(name, decode_path):
    """The same binary and inputs give the same output and index bytes in this process
    (twice) and in a fresh one (the two full-size configurations: default launch shape only)."""
    import subprocess
    import sys as _sys
    from tests.determinism_child import digest
    if name in ("C3", "C4a") and decode_path != "auto":
        pytest.skip("full-size configurations on the default launch shape only")
    k3, k4, k1 = ds.ds_tune_get(3), ds.ds_tune_get(4), ds.ds_tune_get(1)
    here = digest(name, k3, k4, k1)
    assert digest(name, k3, k4, k1) == here
    ds.ds_tune_set(3, k3); ds.ds_tune_set(4, k4); ds.ds_tune_set(1, k1)
    child = os.path.join(os.path.dirname(os.path.abspath(__file__)), "determinism_child.py")
    res = subprocess.run([_sys.executable, child, name, str(k3), str(k4), str(k1)], capture_output=True, text=True,
                         timeout=240)
    assert res.returncode == 0, res.stderr[-2000:]
    there = [ln.split()[1] for ln in res.stdout.splitlines() if ln.startswith("digest ")]
    assert there == [here]


# ---------------------------------------------------------------- determinism across tuning-independent reruns
def test_run_to_run_bytes_identical_c1_many_times():
    w = WORKLOADS["C1"]
    t = make_layer_numpy(w)
    case = Case(t["q"], t["K"], t["V"], outlier_channels(w.Hkv, w.d), w.L, w.k)
    case.gpu_build_label()
    first = None
    for _ in range(5):
        out, idx = case.gpu_sparse()
        blob = out.tobytes() + idx.tobytes()
        first = first or blob
        assert blob == first
