"""The entry point that allocates nothing (ds_sparse_decode_static) against
ds_sparse_decode on the same inputs, through the C ABI: two calls in a row on the
library's own scratch array, the second with a smaller input of another shape, then
the first shape again.  Same kernels in the same launch shapes, so outputs and index
lists must be the same bytes; the index lists are also checked against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2408_07092_amd as ds
from oracle import ds_oracle as O
from tests.parity_util import Case, check_output
from workloads import Workload, make_layer_numpy

pytestmark = pytest.mark.gpu


def _case(B, Hq, Hkv, L, L_max, r, k, seed):
    w = Workload("t", B, Hq, Hkv, 128, L, r, k, 1)
    t = make_layer_numpy(w, layer=seed, L_max=L_max)
    rng = np.random.default_rng(seed)
    ch = np.stack([np.sort(rng.permutation(128)[:r]) for _ in range(Hkv)]).astype(np.int32)
    case = Case(t["q"], t["K"], t["V"], ch, L, k)
    case.gpu_build_label()
    return case


def _static(case, want_idx=True):
    out = torch.full((case.B, case.Hq, case.d), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((case.B, case.Hkv, case.k), -7, dtype=torch.int32, device="cuda") if want_idx else None
    ds.ds_sparse_decode_static(case.q, case.label, case.K, case.V, case.ch, out, idx, case.shape)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (idx.cpu().numpy() if want_idx else None)


def test_static_scratch_decode_matches_workspace_decode():
    assert ds.ds_static_scratch_bytes() == 32 << 20
    ds.ds_static_init()
    big = _case(2, 4, 4, 40000, 40000, 8, 2500, seed=5)      # several workgroups per unit, one launch
    small = _case(1, 8, 2, 3001, 3008, 16, 190, seed=6)      # a query group, one workgroup per unit
    mid = _case(1, 2, 2, 9000, 9000, 5, 560, seed=7)         # odd r: separate scoring launch
    for name, case in (("big", big), ("small", small), ("mid", mid), ("big again", big)):
        print("static-scratch decode:", name, flush=True)
        ref_out, ref_idx = case.gpu_sparse()
        out, idx = _static(case)
        assert np.array_equal(idx, ref_idx), f"{name}: index lists differ"
        assert out.tobytes() == ref_out.tobytes(), f"{name}: outputs differ"
        lab = O.build_label(case.K_h, case.ch_h, case.L)
        o64, i32, _, _ = O.sparse_decode(case.q_h, lab, case.K_h, case.V_h, case.ch_h, case.L, case.k,
                                         precision=32, want_scores=True)
        assert np.array_equal(idx, i32), f"{name}: index lists differ from the oracle"
        check_output(out, O.attend_idx(case.q_h, case.K_h, case.V_h, idx), name)
        out2, _ = _static(case, want_idx=False)
        assert out2.tobytes() == out.tobytes(), f"{name}: output depends on idx_out"


def test_static_scratch_refuses_shapes_beyond_its_size():
    """A shape whose scratch layout exceeds the array is refused before anything is enqueued."""
    shp = ds.shape(1, 32, 32, 128, 262144, 262144, 8, 16384)
    x = torch.zeros(1 << 16, dtype=torch.float16, device="cuda")
    ch = torch.zeros((32, 8), dtype=torch.int32, device="cuda")
    out = torch.full((1, 32, 128), 3.0, dtype=torch.float32, device="cuda")
    with pytest.raises(ds.DsError) as e:
        ds.ds_sparse_decode_static(x, x, x, x, ch, out, None, shp)
    assert e.value.status == ds.DS_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (out == 3.0).all()
