"""Helpers of the GPU parity tests: run the HIP path through the binding, run the
CPU oracle on the same inputs, and compare to the acceptance bar.

Acceptance bar (written out here so the tests state it):
  * label cache, index lists: bit-exact.  Index sets are compared twice:
      - against the oracle selecting on binary32 scores in the library's stated
        order: must be identical;
      - against the oracle selecting on float64 scores: identical except inside
        the near-tie band |s - tau_k| <= 1e-3 * max(|s|, |tau_k|) around the
        k-th score tau_k; everything above the band must be selected, nothing
        below it may be.
  * outputs (fp16 inputs, fp32 accumulation): max |y - y_ref| <= 2e-3 and
    ||y - y_ref||_2 / ||y_ref||_2 <= 1e-2 per (batch, head) row, y_ref = oracle
    in float64 (on the library's index set if that differs inside the band).
  * run-to-run: bytes identical.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2408_07092_amd as ds
from oracle import ds_oracle as O

ABS_TOL = 2e-3
REL_TOL = 1e-2
BAND = 1e-3


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


GUARD = 256  # bytes of canary on either side of a guarded buffer


class Guarded:
    """A device buffer between two canary bands: `view` is what the library gets; check()
    asserts that nothing was written outside it."""

    def __init__(self, nbytes, dtype, shape=None, fill=None):
        self.raw = torch.full((nbytes + 2 * GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        inner = self.raw[GUARD:GUARD + nbytes]
        self.view = inner.view(dtype) if shape is None else inner.view(dtype).view(shape)
        if fill is not None:
            self.view.fill_(fill)

    def check(self, what):
        lo, hi = self.raw[:GUARD], self.raw[-GUARD:]
        assert bool((lo == 0xA5).all()) and bool((hi == 0xA5).all()), f"{what}: written outside the buffer"


def guarded_workspace(shape):
    """Cleared workspace of exactly ds_workspace_bytes() between canary bands."""
    n = ds.ds_workspace_bytes(shape)
    g = Guarded(n, torch.uint8)
    ds.ds_workspace_init(g.view)
    torch.cuda.synchronize()
    return g


class Case:
    """Device tensors + shape for one layer; host copies for the oracle."""

    def __init__(self, q, K, V, channels, L, k):
        self.q_h, self.K_h, self.V_h = q, K, V
        self.ch_h = np.ascontiguousarray(channels, dtype=np.int32)
        self.B, self.Hq, self.d = q.shape
        _, self.Hkv, self.L_max, _ = K.shape
        self.L, self.k, self.r = L, k, self.ch_h.shape[1]
        self.q, self.K, self.V = to_dev(q), to_dev(K), to_dev(V)
        self.ch = to_dev(self.ch_h)
        self.shape = ds.shape(self.B, self.Hq, self.Hkv, self.d, L, self.L_max, self.r, k)
        self.label = torch.zeros((self.B, self.Hkv, self.L_max, self.r), dtype=torch.float16, device="cuda")
        self._ws_guard = guarded_workspace(self.shape)
        self.ws = self._ws_guard.view

    @classmethod
    def from_torch(cls, t, channels, L, k):
        """t: dict of device tensors (q, K, V) from the torch generator."""
        self = cls.__new__(cls)
        self.q, self.K, self.V = t["q"], t["K"], t["V"]
        self.q_h, self.K_h, self.V_h = (x.cpu().numpy() for x in (self.q, self.K, self.V))
        self.ch_h = np.ascontiguousarray(channels, dtype=np.int32)
        self.B, self.Hq, self.d = self.q_h.shape
        _, self.Hkv, self.L_max, _ = self.K_h.shape
        self.L, self.k, self.r = L, k, self.ch_h.shape[1]
        self.ch = to_dev(self.ch_h)
        self.shape = ds.shape(self.B, self.Hq, self.Hkv, self.d, L, self.L_max, self.r, k)
        self.label = torch.zeros((self.B, self.Hkv, self.L_max, self.r), dtype=torch.float16, device="cuda")
        self._ws_guard = guarded_workspace(self.shape)
        self.ws = self._ws_guard.view
        return self

    # ---- HIP path
    def gpu_build_label(self):
        ds.ds_build_label(self.K, self.ch, self.label, self.shape)
        torch.cuda.synchronize()
        return self.label.cpu().numpy()

    def _outputs(self, want_idx=True):
        """Output and index buffers between canary bands, pre-filled with values no call writes."""
        out = Guarded(self.B * self.Hq * self.d * 4, torch.float32, (self.B, self.Hq, self.d), float("nan"))
        idx = Guarded(self.B * self.Hkv * self.k * 4, torch.int32, (self.B, self.Hkv, self.k), -7) if want_idx else None
        return out, idx

    def _checked(self, out, idx, what):
        """After a call: nothing outside the output, the index list or the workspace was written
        (the workspace guard only when the call ran on the case's own workspace)."""
        torch.cuda.synchronize()
        out.check(what + " out")
        if idx is not None:
            idx.check(what + " idx_out")
        if self.ws.data_ptr() == self._ws_guard.view.data_ptr():
            self._ws_guard.check(what + " workspace")
        return out.view.cpu().numpy(), (idx.view.cpu().numpy() if idx is not None else None)

    def gpu_sparse(self, want_idx=True):
        out, idx = self._outputs(want_idx)
        ds.ds_sparse_decode(self.q, self.label, self.K, self.V, self.ch, out.view, idx.view if idx else None, self.ws,
                            self.shape)
        return self._checked(out, idx, "ds_sparse_decode")

    def gpu_sparse_nolabel(self):
        out, idx = self._outputs()
        ds.ds_sparse_decode_nolabel(self.q, self.K, self.V, self.ch, out.view, idx.view, self.ws, self.shape)
        return self._checked(out, idx, "ds_sparse_decode_nolabel")

    def gpu_dense(self):
        out, _ = self._outputs(False)
        ds.ds_dense_decode(self.q, self.K, self.V, out.view, self.ws, self.shape)
        return self._checked(out, None, "ds_dense_decode")[0]

    def gpu_select(self):
        out, idx = self._outputs()
        ds.ds_select(self.q, self.label, self.ch, idx.view, self.ws, self.shape)
        return self._checked(out, idx, "ds_select")[1]

    # ---- oracle
    def oracle_label(self):
        return O.build_label(self.K_h, self.ch_h, self.L)

    def oracle_sparse(self, label_h, precision):
        return O.sparse_decode(self.q_h, label_h, self.K_h, self.V_h, self.ch_h, self.L, self.k,
                               precision=precision, want_scores=True)


def check_output(y, y_ref, what=""):
    """Both required: max abs error <= 2e-3, per-row relative L2 error <= 1e-2."""
    y = np.asarray(y, dtype=np.float64)
    assert np.isfinite(y).all(), f"{what}: non-finite output"
    err = np.abs(y - y_ref)
    assert err.max() <= ABS_TOL, f"{what}: max abs err {err.max():.3e} > {ABS_TOL}"
    num = np.sqrt(((y - y_ref) ** 2).sum(-1))
    den = np.sqrt((y_ref ** 2).sum(-1))
    rel = num / np.maximum(den, 1e-30)
    assert rel.max() <= REL_TOL, f"{what}: rel err {rel.max():.3e} > {REL_TOL}"
    return float(err.max()), float(rel.max())


def check_index_structure(idx, L, k):
    """Shape rules of an index list: k_eff ascending distinct in-range entries, then -1."""
    k_eff = min(k, L)
    head, tail = idx[..., :k_eff], idx[..., k_eff:]
    assert (tail == -1).all(), "tail beyond k_eff must be -1"
    assert (head >= 0).all() and (head < L).all(), "index out of range"
    if k_eff > 1:
        assert (np.diff(head, axis=-1) > 0).all(), "indices must be strictly ascending"


def check_index_band(idx_gpu, scores64, sorted64, L, k):
    """Float64-oracle comparison with the near-tie band.  Returns the number of
    units whose set differs from the float64 oracle's (all inside the band)."""
    B, Hkv, _ = idx_gpu.shape
    k_eff = min(k, L)
    differing = 0
    for b in range(B):
        for h in range(Hkv):
            s, srt = scores64[b, h], sorted64[b, h]
            tau = srt[k_eff - 1]
            in_band = np.abs(s - tau) <= BAND * np.maximum(np.abs(s), abs(tau))
            must = (s > tau) & ~in_band
            never = (s < tau) & ~in_band
            chosen = np.zeros(L, dtype=bool)
            chosen[idx_gpu[b, h, :k_eff]] = True
            assert chosen.sum() == k_eff
            assert chosen[must].all(), f"unit ({b},{h}): a token above the band was not selected"
            assert not chosen[never].any(), f"unit ({b},{h}): a token below the band was selected"
            want = np.zeros(L, dtype=bool)
            order = np.lexsort((np.arange(L), -s))[:k_eff]
            want[order] = True
            if (want != chosen).any():
                differing += 1
                if k_eff < L:
                    nxt = srt[k_eff]
                    assert abs(tau - nxt) <= BAND * max(abs(tau), abs(nxt)), \
                        f"unit ({b},{h}): sets differ although the k-th and (k+1)-th scores are separated"
    return differing


def check_decode_against_both_oracles(idx_gpu, out_gpu, q, label, K, V, ch, L, k, what=""):
    """Index list and output of one decode against the oracle in both of its modes: identical
    to the selection on binary32 scores in the library's stated order, identical to the float64
    definition except inside the near-tie band, output within the bar of the float64 oracle
    (evaluated on the library's set if that differs inside the band)."""
    check_index_structure(idx_gpu, L, k)
    _, idx32 = O.sparse_decode(q, label, K, V, ch, L, k, precision=32)
    assert np.array_equal(idx_gpu, idx32), f"{what}: index sets differ from the binary32-order oracle"
    out64, _, sc64, srt64 = O.sparse_decode(q, label, K, V, ch, L, k, precision=64, want_scores=True)
    differing = check_index_band(idx_gpu, sc64, srt64, L, k)
    ref = out64 if differing == 0 else O.attend_idx(q, K, V, idx_gpu)
    return check_output(out_gpu, ref, what)


def full_parity(case: Case, check_dense=True, what=""):
    """Every stage of the path against the oracle; returns a small report dict."""
    # a0: label cache
    lab_gpu = case.gpu_build_label()
    lab_ref = case.oracle_label()
    assert np.array_equal(lab_gpu.view(np.uint16)[:, :, :case.L], lab_ref.view(np.uint16)[:, :, :case.L]), \
        f"{what}: label cache differs"
    # a1-a4
    out_gpu, idx_gpu = case.gpu_sparse()
    check_index_structure(idx_gpu, case.L, case.k)
    out32, idx32, _, _ = case.oracle_sparse(lab_ref, 32)
    assert np.array_equal(idx_gpu, idx32), f"{what}: index sets differ from the binary32-order oracle"
    out64, idx64, sc64, srt64 = case.oracle_sparse(lab_ref, 64)
    differing = check_index_band(idx_gpu, sc64, srt64, case.L, case.k)
    ref = out64 if differing == 0 else O.attend_idx(case.q_h, case.K_h, case.V_h, idx_gpu)
    abs_err, rel_err = check_output(out_gpu, ref, what + " sparse")
    # without idx_out the output must be the same bytes
    out_gpu2, _ = case.gpu_sparse(want_idx=False)
    assert out_gpu2.tobytes() == out_gpu.tobytes(), f"{what}: output depends on idx_out / not reproducible"
    # ds_select alone gives the same list
    assert np.array_equal(case.gpu_select(), idx_gpu), f"{what}: ds_select differs from ds_sparse_decode"
    # scoring straight from the K rows (no label cache): same selection as the binary32-order
    # oracle, output to the same bar
    out_nl, idx_nl = case.gpu_sparse_nolabel()
    check_index_structure(idx_nl, case.L, case.k)
    assert np.array_equal(idx_nl, idx32), f"{what}: no-label index sets differ from the binary32-order oracle"
    check_output(out_nl, ref, what + " sparse, no label cache")
    rep = {"abs_err": abs_err, "rel_err": rel_err, "units_differing_in_band": differing}
    if check_dense:
        d_gpu = case.gpu_dense()
        d_ref = O.dense_decode(case.q_h, case.K_h, case.V_h, case.L)
        rep["dense_abs_err"], rep["dense_rel_err"] = check_output(d_gpu, d_ref, what + " dense")
        assert case.gpu_dense().tobytes() == d_gpu.tobytes(), f"{what}: dense not reproducible"
    return rep
