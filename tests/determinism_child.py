"""Child process of the cross-process determinism test: runs one seeded decode
through the library and prints the SHA-256 of the output and index bytes.
Usage: python determinism_child.py <workload> <knob3> <knob4> <knob1>"""
import hashlib
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def digest(name, knob3, knob4, knob1=0):
    import torch

    import paper_2408_07092_amd as ds
    from workloads import WORKLOADS, make_layer_numpy, outlier_channels

    w = WORKLOADS[name] if name in WORKLOADS else WORKLOADS["C1"].scaled(Hq=8, Hkv=8, L=12000, k=700)
    ds.ds_tune_set(3, knob3)
    ds.ds_tune_set(4, knob4)
    ds.ds_tune_set(1, knob1)
    t = make_layer_numpy(w)
    q, K, V = (torch.from_numpy(t[n]).cuda() for n in ("q", "K", "V"))
    ch = torch.from_numpy(outlier_channels(w.Hkv, w.d)).cuda()
    shp = ds.shape(w.B, w.Hq, w.Hkv, w.d, w.L, w.L, w.r, w.k)
    label = torch.empty((w.B, w.Hkv, w.L, w.r), dtype=torch.float16, device="cuda")
    ds.ds_build_label(K, ch, label, shp)
    ws = ds.ds_workspace_alloc(shp)
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.B, w.Hkv, w.k), dtype=torch.int32, device="cuda")
    ds.ds_sparse_decode(q, label, K, V, ch, out, idx, ws, shp)
    torch.cuda.synchronize()
    ds.ds_tune_set(3, 0)
    ds.ds_tune_set(4, 0)
    ds.ds_tune_set(1, 0)
    return hashlib.sha256(out.cpu().numpy().tobytes() + idx.cpu().numpy().tobytes()).hexdigest()


if __name__ == "__main__":
    print("digest", digest(sys.argv[1], int(sys.argv[2]), int(sys.argv[3]), int(sys.argv[4])))
