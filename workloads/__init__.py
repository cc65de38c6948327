"""Seeded synthetic decode-attention workloads.

Shared by the CPU oracle's tests and by the HIP path's tests and bench: this
module only draws inputs.  It holds none of the method's arithmetic (no
scoring, selection, softmax or calibration).

The tensors stand in for Llama-2-7B / Llama-2-70B / Mixtral-8x7B KV caches
(public attention shapes; no trained weights or datasets are used).  Values
follow the static-outlier-channel structure the method relies on (Sec. 1 and
Sec. 4.1 of the paper): K, V, q ~ N(0,1); in every (layer, KV head) a fixed
seeded set of 8 channels is multiplied by 8 in both q and K before the fp16
cast.  V is not scaled.  The set does not depend on batch or token.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED = 20240807
N_OUTLIER = 8
OUTLIER_SCALE = 8.0


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    L: int
    r: int
    k: int
    n_layers: int
    note: str = ""

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def units(self) -> int:
        return self.B * self.Hkv

    def algorithmic_bytes(self) -> int:
        """Bytes one layer of the sparse path must read (Sec. 5.3 IO model):
        label stream L*r fp16 plus k full K and V rows, per (batch, KV head)."""
        return self.units * (self.L * self.r * 2 + self.k * self.d * 2 * 2)

    def dense_bytes(self) -> int:
        return self.units * 4 * self.L * self.d

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "C1": Workload("C1", 1, 32, 32, 128, 4096, 8, 256, 1, "single layer, small"),
    "C2": Workload("C2", 8, 32, 32, 128, 16384, 16, 1024, 32, "Llama-2-7B-shaped, batch 8"),
    "C3": Workload("C3", 1, 32, 32, 128, 65536, 8, 4096, 32, "Llama-2-7B-shaped, L=64K (headline)"),
    "C4a": Workload("C4a", 16, 64, 8, 128, 32768, 8, 2048, 80, "Llama-2-70B-shaped GQA, group 8"),
    "C4b": Workload("C4b", 16, 32, 8, 128, 32768, 8, 2048, 32, "Mixtral-shaped GQA, group 4"),
    # two corners of the batch x length grid of the paper's label-cache ablation table (appendix):
    "A1": Workload("A1", 32, 32, 32, 128, 2048, 8, 128, 32, "ablation grid corner: batch 32, 2K tokens"),
    "A2": Workload("A2", 32, 32, 32, 128, 8192, 8, 512, 32, "ablation grid corner: batch 32, 8K tokens"),
    "C5": Workload("C5", 1, 32, 32, 128, 262144, 8, 16384, 32, "offload-style, K/V in pinned host memory"),
}


def _rng(seed: int, layer: int, tag: int) -> np.random.Generator:
    return np.random.default_rng([seed, layer, tag])


def outlier_channels(Hkv: int, d: int, layer: int = 0, seed: int = SEED) -> np.ndarray:
    """[Hkv, 8] int32, ascending: the static outlier channels of each KV head."""
    rng = _rng(seed, layer, 1)
    return np.stack([np.sort(rng.choice(d, size=N_OUTLIER, replace=False))
                     for _ in range(Hkv)]).astype(np.int32)


def channel_scale(Hkv: int, d: int, layer: int = 0, seed: int = SEED) -> np.ndarray:
    """[Hkv, d] float32: 8 on the outlier channels of the head, 1 elsewhere."""
    s = np.ones((Hkv, d), dtype=np.float32)
    out = outlier_channels(Hkv, d, layer, seed)
    for h in range(Hkv):
        s[h, out[h]] = OUTLIER_SCALE
    return s


def make_layer_numpy(w: Workload, layer: int = 0, seed: int = SEED, L_max: int | None = None):
    """One layer's decode inputs on the host: dict of fp16 numpy arrays
    q [B,Hq,d], K,V [B,Hkv,L_max,d] (tokens >= L are zero)."""
    L_max = w.L if L_max is None else L_max
    assert L_max >= w.L
    scale = channel_scale(w.Hkv, w.d, layer, seed)
    K = np.zeros((w.B, w.Hkv, L_max, w.d), dtype=np.float16)
    V = np.zeros((w.B, w.Hkv, L_max, w.d), dtype=np.float16)
    rk, rv, rq = _rng(seed, layer, 2), _rng(seed, layer, 3), _rng(seed, layer, 4)
    for b in range(w.B):
        for h in range(w.Hkv):
            K[b, h, :w.L] = (rk.standard_normal((w.L, w.d), dtype=np.float32) * scale[h]).astype(np.float16)
            V[b, h, :w.L] = rv.standard_normal((w.L, w.d), dtype=np.float32).astype(np.float16)
    q = rq.standard_normal((w.B, w.Hq, w.d), dtype=np.float32)
    q = (q * np.repeat(scale, w.G, axis=0)[None]).astype(np.float16)
    return {"q": q, "K": K, "V": V}


def make_calibration_numpy(w: Workload, layer: int = 0, seed: int = SEED, N: int = 512):
    """N extra (q, k) sample rows drawn like the layer: q_calib [N,Hq,d],
    k_calib [N,Hkv,d] fp16, for the offline calibration (Sec. 4.1)."""
    scale = channel_scale(w.Hkv, w.d, layer, seed)
    rng = _rng(seed, layer, 5)
    qc = rng.standard_normal((N, w.Hq, w.d), dtype=np.float32) * np.repeat(scale, w.G, axis=0)[None]
    kc = rng.standard_normal((N, w.Hkv, w.d), dtype=np.float32) * scale[None]
    return qc.astype(np.float16), kc.astype(np.float16)


def make_layer_torch(w: Workload, device, layer: int = 0, seed: int = SEED,
                     L_max: int | None = None, kv_device=None, pin_kv: bool = False):
    """Same recipe drawn with torch's generator on `device` (fast enough for the
    full-size caches).  Returns dict of fp16 torch tensors q, K, V.  The numpy
    and torch generators give different streams of the same distribution; a
    parity test copies the torch tensors to the host for the oracle.
    With pin_kv the K and V tensors are returned in pinned host memory."""
    import torch

    L_max = w.L if L_max is None else L_max
    g = torch.Generator(device=device)
    g.manual_seed(seed + 1000003 * layer + 17)
    scale = torch.from_numpy(channel_scale(w.Hkv, w.d, layer, seed)).to(device)
    shape = (w.B, w.Hkv, L_max, w.d)
    if pin_kv:
        K = torch.empty(shape, dtype=torch.float16, pin_memory=True)
        V = torch.empty(shape, dtype=torch.float16, pin_memory=True)
    else:
        K = torch.zeros(shape, dtype=torch.float16, device=device)
        V = torch.zeros(shape, dtype=torch.float16, device=device)
    # one (batch) slab at a time keeps the fp32 temporaries small
    for b in range(w.B):
        kb = torch.randn((w.Hkv, w.L, w.d), generator=g, device=device, dtype=torch.float32)
        kb.mul_(scale[:, None, :])
        K[b, :, :w.L].copy_(kb.to(torch.float16))
        vb = torch.randn((w.Hkv, w.L, w.d), generator=g, device=device, dtype=torch.float32)
        V[b, :, :w.L].copy_(vb.to(torch.float16))
        if pin_kv and L_max > w.L:
            K[b, :, w.L:].zero_(); V[b, :, w.L:].zero_()
    q = torch.randn((w.B, w.Hq, w.d), generator=g, device=device, dtype=torch.float32)
    q = (q * scale.repeat_interleave(w.G, dim=0)[None]).to(torch.float16)
    return {"q": q, "K": K, "V": V}
