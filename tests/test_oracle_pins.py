"""Pins for the CPU oracle: each test fixes a part of oracle/ds_oracle.c against
something other than the oracle itself -- numpy float64 library routines,
brute force on tiny inputs, closed forms, invariants, and a hand-derived
fixture.  A plausible slip (dropped term, wrong sign/index, transposed operand,
missing 1/sqrt(d), wrong tie rule) fails at least one of them.  CPU only."""
import json
import os

import numpy as np
import pytest

from oracle import ds_oracle as O
from workloads import WORKLOADS, make_calibration_numpy, make_layer_numpy, outlier_channels

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def np_dense(q, K, V, L):
    """Sec. 2.1 with numpy float64 matmul/exp, per q head (library routine pin)."""
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.empty((B, Hq, d))
    for b in range(B):
        for hq in range(Hq):
            k = K[b, hq // G, :L].astype(np.float64)
            v = V[b, hq // G, :L].astype(np.float64)
            s = k @ q[b, hq].astype(np.float64) / np.sqrt(d)
            p = np.exp(s - s.max())
            out[b, hq] = (p / p.sum()) @ v
    return out


def small_case(B=2, Hq=4, Hkv=4, d=16, L=37, L_max=40, seed=0, ints=False):
    rng = np.random.default_rng(seed)
    if ints:
        draw = lambda *s: rng.integers(-3, 4, size=s).astype(np.float16)
    else:
        draw = lambda *s: rng.standard_normal(s).astype(np.float16)
    q = draw(B, Hq, d)
    K = np.zeros((B, Hkv, L_max, d), np.float16); K[:, :, :L] = draw(B, Hkv, L, d)
    V = np.zeros((B, Hkv, L_max, d), np.float16); V[:, :, :L] = draw(B, Hkv, L, d)
    return q, K, V


# ---------------------------------------------------------------- fp16 widening
def test_half_to_double_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = O.half_to_double(h)
    want = h.astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- dense formula
@pytest.mark.parametrize("G", [1, 2, 4])
def test_dense_matches_numpy_float64(G):
    q, K, V = small_case(Hq=4 * G, Hkv=4, seed=G)
    got = O.dense_decode(q, K, V, 37)
    np.testing.assert_allclose(got, np_dense(q, K, V, 37), rtol=1e-12, atol=1e-13)


def test_dense_hand_derived_fixture():
    fx = json.load(open(os.path.join(GOLDEN, "logistic_two_token.json")))
    q = np.array(fx["q"], np.float16).reshape(1, 1, 4)
    K = np.array(fx["K"], np.float16).reshape(1, 1, 2, 4)
    V = np.array(fx["V"], np.float16).reshape(1, 1, 2, 4)
    got = O.dense_decode(q, K, V, 2)[0, 0]
    np.testing.assert_allclose(got, fx["y"], rtol=0, atol=1e-14)
    # Algorithm 1 with k = S and two label channels reaches the same value
    ch = np.array([[0, 1]], np.int32)
    lab = O.build_label(K, ch, 2)
    out, idx = O.sparse_decode(q, lab, K, V, ch, 2, 2)
    np.testing.assert_allclose(out[0, 0], fx["y"], rtol=0, atol=1e-14)
    assert idx.tolist() == [[[0, 1]]]


def test_dense_closed_forms():
    rng = np.random.default_rng(5)
    d, L = 8, 11
    q = rng.standard_normal((1, 1, d)).astype(np.float16)
    V = rng.standard_normal((1, 1, L, d)).astype(np.float16)
    # all keys equal -> uniform weights -> y = mean of V rows
    K = np.tile(rng.standard_normal((1, 1, 1, d)).astype(np.float16), (1, 1, L, 1))
    np.testing.assert_allclose(O.dense_decode(q, K, V, L)[0, 0],
                               V[0, 0].astype(np.float64).mean(0), rtol=1e-13, atol=1e-14)
    # one key = 64*q, the rest 0 -> that token's weight -> 1
    K = np.zeros((1, 1, L, d), np.float16); K[0, 0, 7] = (64 * q[0, 0].astype(np.float32)).astype(np.float16)
    qq = float((q.astype(np.float64) ** 2).sum())
    y = O.dense_decode(q, K, V, L)[0, 0]
    w_other = (L - 1) * np.exp(-64 * qq / np.sqrt(d))
    np.testing.assert_allclose(y, V[0, 0, 7].astype(np.float64), atol=10 * w_other + 1e-12)
    # tokens beyond L are ignored
    K2 = rng.standard_normal((1, 1, L, d)).astype(np.float16)
    np.testing.assert_allclose(O.dense_decode(q, K2, V, 6), np_dense(q, K2, V, 6), rtol=1e-12)


def test_dense_has_inverse_sqrt_d_scale_and_shift_invariance():
    # softmax logits must be q.k/sqrt(d): with d = 4, q.k in {2 ln-ish}. Use a
    # 2-token case whose weights are exactly logistic(q.k0/2 - q.k1/2).
    q = np.array([[[4, 0, 0, 0]]], np.float16)
    K = np.array([[[[1, 0, 0, 0], [0.5, 0, 0, 0]]]], np.float16)   # logits 2 and 1
    V = np.array([[[[1, 0, 0, 0], [0, 1, 0, 0]]]], np.float16)
    y = O.dense_decode(q, K, V, 2)[0, 0]
    p0 = 1.0 / (1.0 + np.exp(-1.0))
    np.testing.assert_allclose(y[:2], [p0, 1 - p0], atol=1e-15)
    # adding the same vector along q to every key shifts all logits equally
    K2 = K.copy(); K2[..., 0] += 2
    np.testing.assert_allclose(O.dense_decode(q, K2, V, 2)[0, 0], y, atol=1e-15)


# ---------------------------------------------------------------- label cache
def test_label_is_exact_channel_copy_and_append_equals_build():
    q, K, V = small_case(d=16, L=37, L_max=40, seed=3)
    rng = np.random.default_rng(0)
    ch = np.stack([rng.permutation(16)[:5] for _ in range(4)]).astype(np.int32)  # unsorted order allowed
    lab = O.build_label(K, ch, 37)
    for h in range(4):
        assert np.array_equal(lab[:, h, :37].view(np.uint16), K[:, h, :37][..., ch[h]].view(np.uint16))
    assert not lab[:, :, 37:].any()
    lab2 = O.build_label(K, ch, 30)
    O.label_write(K, ch, lab2, 30, 4)
    O.label_write(K, ch, lab2, 34, 3)
    assert np.array_equal(lab.view(np.uint16), lab2.view(np.uint16))


def test_append_kv_equals_cache_built_in_one_go():
    """Appending the last tokens' rows to a shorter cache gives the bytes of the
    cache that held them from the start, label cache included; decode results agree."""
    q, K, V = small_case(d=16, L=37, L_max=40, seed=5)
    ch = np.stack([np.sort(np.random.default_rng(h).permutation(16)[:4]) for h in range(4)]).astype(np.int32)
    lab = O.build_label(K, ch, 37)
    K2, V2 = K.copy(), V.copy()
    K2[:, :, 30:] = 0; V2[:, :, 30:] = 0
    lab2 = O.build_label(K2, ch, 30)
    O.append_kv(K[:, :, 30:35].copy(), V[:, :, 30:35].copy(), K2, V2, ch, lab2, 30)
    O.append_kv(K[:, :, 35:37].copy(), V[:, :, 35:37].copy(), K2, V2, ch, lab2, 35)
    for a, b in ((K, K2), (V, V2), (lab, lab2)):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    kv = O.interleave_kv(K, V)
    assert kv.shape == K.shape[:3] + (2, 16)
    assert np.array_equal(kv[:, :, :, 0].view(np.uint16), K.view(np.uint16))
    assert np.array_equal(kv[:, :, :, 1].view(np.uint16), V.view(np.uint16))


def test_predict_query_hand_case_identity_and_linearity():
    # 2 x 3 projection written out: q0 = 1*1 + 2*(-2) + 0.5*4 = -1, q1 = 0*1 + (-1)*(-2) + 3*4 = 14
    Wq = np.array([[1, 2, 0.5], [0, -1, 3]], np.float16)
    x = np.array([[1, -2, 4]], np.float16)
    assert O.predict_query(x, Wq).tolist() == [[-1.0, 14.0]]
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 16)).astype(np.float16)
    assert np.array_equal(O.predict_query(x, np.eye(16, dtype=np.float16)), x)   # identity projection
    W = rng.integers(-2, 3, size=(5, 16)).astype(np.float16)
    xi = rng.integers(-3, 4, size=(2, 16)).astype(np.float16)                    # integers: exact in fp16
    got = O.predict_query(np.stack([xi[0], xi[1], xi[0] + xi[1]]), W).astype(np.float64)
    assert np.array_equal(got[2], got[0] + got[1])
    assert O.predict_query(x, W).shape == (3, 5)                                 # rows of Wq are output features


# ---------------------------------------------------------------- 4-bit label cache
def _unpack_q4(codes, r):
    """numpy view of the packed codes as int [.., r] (independent of the oracle's unpacking)."""
    out = np.empty(codes.shape[:-1] + (r,), dtype=np.int64)
    for j in range(r):
        nib = (codes[..., j // 8] >> np.uint32(4 * (j % 8))) & np.uint32(15)
        out[..., j] = np.where(nib >= 8, nib.astype(np.int64) - 16, nib.astype(np.int64))
    return out


def test_q4_hand_case_codes_and_packing():
    # one unit, r = 3 channels (5, 0, 2), four tokens, amax = 7, 3.5, 0 -> steps 1, 0.5, 0
    K = np.zeros((1, 1, 5, 8), np.float16)
    K[0, 0, :4, 5] = [7, -7, 2.5, -3.5]        # x*inv = x: 2.5 -> 2 and -3.5 -> -4 (half to even)
    K[0, 0, :4, 0] = [3.5, 0.25, -0.75, 1.0]   # x*inv = 2x: 7, 0.5 -> 0, -1.5 -> -2, 2
    ch = np.array([[5, 0, 2]], np.int32)
    codes, amax = O.build_label_q4(K, ch, 4)
    assert amax.tolist() == [[[7.0, 3.5, 0.0]]]
    want = np.array([[7, 7, 0], [-7, 0, 0], [2, -2, 0], [-4, 2, 0]])
    assert np.array_equal(_unpack_q4(codes, 3)[0, 0, :4], want)
    assert codes.shape == (1, 1, 5, 1) and not codes[0, 0, 4].any()
    # packing: channel j in bits [4j, 4j+4), two's complement; unused nibbles zero
    assert int(codes[0, 0, 1, 0]) == ((-7) & 15) | (0 << 4)
    assert int(codes[0, 0, 3, 0]) == ((-4) & 15) | (2 << 4)
    # an appended token beyond amax saturates at -8 / 7 under the frozen amax
    K[0, 0, 4, 5], K[0, 0, 4, 0] = -100.0, 100.0
    O.label_q4_write(K, ch, amax, codes, 4, 1)
    assert _unpack_q4(codes, 3)[0, 0, 4].tolist() == [-8, 7, 0]


@pytest.mark.parametrize("r", [1, 8, 11, 16])
def test_q4_quantiser_error_bound_range_and_scale_equivariance(r):
    q, K, V = small_case(d=32, L=61, L_max=64, seed=r)
    rng = np.random.default_rng(r)
    ch = np.stack([rng.permutation(32)[:r] for _ in range(4)]).astype(np.int32)
    codes, amax = O.build_label_q4(K, ch, 61)
    c = _unpack_q4(codes, r)
    assert c.min() >= -8 and c.max() <= 7
    lab = np.stack([K[:, h][..., ch[h]] for h in range(4)], axis=1).astype(np.float64)   # [B,Hkv,L_max,r]
    assert np.array_equal(amax, np.abs(lab[:, :, :61]).max(axis=2).astype(np.float32))
    step = (amax / np.float32(7.0)).astype(np.float64)[:, :, None, :]
    err = np.abs(c[:, :, :61] * step - lab[:, :, :61])
    assert (err <= 0.5 * step * (1 + 1e-6)).all()          # nearest code; never further than half a step
    assert (np.abs(c[:, :, :61]).max(axis=2) == 7).all()    # the largest element of a channel maps to +-7
    assert not codes[:, :, 61:].any()
    # doubling K doubles amax and leaves every code unchanged (power-of-two scaling is exact)
    codes2, amax2 = O.build_label_q4((K * np.float16(2)).astype(np.float16), ch, 61)
    assert np.array_equal(amax2, amax * 2) and np.array_equal(codes2, codes)
    # append == build
    codes3 = np.zeros_like(codes)
    O.label_q4_write(K, ch, amax, codes3, 0, 40)
    O.label_q4_write(K, ch, amax, codes3, 40, 21)
    assert np.array_equal(codes3, codes)


@pytest.mark.parametrize("G", [1, 4])
def test_q4_scores_equal_numpy_on_dequantised_labels_and_binary32_order(G):
    q, K, V = small_case(Hq=4 * G, d=32, L=50, L_max=50, seed=7 + G)
    ch = np.stack([np.sort(np.random.default_rng(h).permutation(32)[:8]) for h in range(4)]).astype(np.int32)
    codes, amax = O.build_label_q4(K, ch, 50)
    c = _unpack_q4(codes, 8).astype(np.float64)
    step32 = amax / np.float32(7.0)
    deq = c * step32.astype(np.float64)[:, :, None, :]
    s64 = O.scores_q4(q, codes, amax, ch, 50, precision=64)
    s32 = O.scores_q4(q, codes, amax, ch, 50, precision=32)
    for b in range(2):
        for h in range(4):
            qg = q[b, h * G:(h + 1) * G][:, ch[h]].astype(np.float64)           # [G, r]
            np.testing.assert_allclose(s64[b, h], deq[b, h] @ qg.sum(0), rtol=1e-12, atol=1e-12)
            # binary32 mode: w_j = (sum_g q_g[C_j]) * step_j in float32, then sequential fma
            w = np.zeros(8, np.float32)
            for g in range(G):
                w = w + q[b, h * G + g][ch[h]].astype(np.float32)
            w = w * step32[b, h]
            for t in (0, 17, 49):
                acc = np.float32(0)
                for j in range(8):   # products of a float32 and a small integer: fma == exact product, then one rounding
                    acc = np.float32(np.float64(w[j]) * c[b, h, t, j] + np.float64(acc))
                assert s32[b, h, t] == np.float64(acc)


def test_q4_sparse_decode_is_topk_of_q4_scores_then_exact_attention_and_k_ge_L_is_dense():
    q, K, V = small_case(d=32, L=64, L_max=64, seed=21)
    ch = np.stack([np.sort(np.random.default_rng(h + 9).permutation(32)[:8]) for h in range(4)]).astype(np.int32)
    codes, amax = O.build_label_q4(K, ch, 64)
    out, idx, sc, srt = O.sparse_decode_q4(q, codes, amax, K, V, ch, 64, 9, want_scores=True)
    assert np.array_equal(sc, O.scores_q4(q, codes, amax, ch, 64))
    for b in range(2):
        for h in range(4):
            want = np.sort(np.lexsort((np.arange(64), -sc[b, h]))[:9])
            assert np.array_equal(idx[b, h], want)
    np.testing.assert_allclose(out, O.attend_idx(q, K, V, idx), rtol=0, atol=0)
    out_all, _ = O.sparse_decode_q4(q, codes, amax, K, V, ch, 64, 64)
    np.testing.assert_allclose(out_all, np_dense(q, K, V, 64), atol=1e-12)


# ---------------------------------------------------------------- approximate scores
def test_scores_hand_case():
    # L = 4, r = 2, channels (3, 1): s_hat[t] = q[3]*K[t,3] + q[1]*K[t,1]
    q = np.array([[[9, 2, 9, -3]]], np.float16)
    K = np.array([[[[7, 1, 7, 1], [7, 0, 7, 2], [7, -4, 7, 0], [7, 0.5, 7, 0.25]]]], np.float16)
    ch = np.array([[3, 1]], np.int32)
    lab = O.build_label(K, ch, 4)
    want = [-3 * 1 + 2 * 1, -3 * 2 + 0, 0 + 2 * -4, -3 * 0.25 + 2 * 0.5]
    for prec in (64, 32):
        assert O.scores(q, lab, ch, 4, prec)[0, 0].tolist() == want


@pytest.mark.parametrize("G", [1, 4])
def test_scores_match_numpy_and_group_sum(G):
    q, K, V = small_case(Hq=2 * G, Hkv=2, d=32, L=50, L_max=50, seed=11)
    rng = np.random.default_rng(1)
    ch = np.stack([np.sort(rng.permutation(32)[:6]) for _ in range(2)]).astype(np.int32)
    lab = O.build_label(K, ch, 50)
    s = O.scores(q, lab, ch, 50, 64)
    for b in range(2):
        for h in range(2):
            qs = sum(q[b, h * G + g].astype(np.float64)[ch[h]] for g in range(G))
            want = K[b, h, :, :][:, ch[h]].astype(np.float64) @ qs
            np.testing.assert_allclose(s[b, h], want, rtol=1e-13, atol=1e-13)
    # binary32 mode differs from the definition only by rounding
    s32 = O.scores(q, lab, ch, 50, 32)
    np.testing.assert_allclose(s32, s, rtol=0, atol=2e-5 * np.abs(s).max())


def test_scores_binary32_mode_is_sequential_fma():
    q, K, V = small_case(Hq=3, Hkv=1, d=16, L=20, L_max=20, seed=2)
    ch = np.array([[1, 4, 5, 9, 15]], np.int32)
    lab = O.build_label(K, ch, 20)
    s32 = O.scores(q, lab, ch, 20, 32)
    qs = np.zeros(5, np.float32)
    for g in range(3):
        qs = (qs + q[0, g][ch[0]].astype(np.float32)).astype(np.float32)
    for t in range(20):
        acc = np.float32(0)
        for j in range(5):
            # fma(a, b, c) with one rounding == round32(exact a*b + c); a*b + c is exact in float64 here
            acc = np.float32(np.float64(qs[j]) * np.float64(lab[0, 0, t, j]) + np.float64(acc))
        assert s32[0, 0, t] == np.float64(acc)


# ---------------------------------------------------------------- argtopk
def brute_topk(s, k):
    order = sorted(range(len(s)), key=lambda t: (-s[t], t))
    return sorted(order[:min(k, len(s))])


def test_topk_equals_bruteforce_full_sort_with_ties():
    rng = np.random.default_rng(7)
    for trial in range(40):
        L = int(rng.integers(1, 65))
        s = rng.integers(-3, 4, size=L).astype(np.float64)      # many exact ties
        if trial % 3 == 0:
            s[rng.integers(0, L)] = -0.0                          # -0 ties with +0
        for k in sorted({1, 2, L // 2 + 1, L, L + 3}):
            idx, srt = O.topk(s, k)
            want = brute_topk(s.tolist(), k)
            assert idx[:len(want)].tolist() == want
            assert (idx[len(want):] == -1).all()
            assert srt.tolist() == sorted(s.tolist(), reverse=True)


def test_topk_invariants_and_nesting():
    rng = np.random.default_rng(8)
    s = rng.standard_normal(500)
    s[100:110] = s[7]                                             # a tie block
    prev = set()
    for k in range(1, 501, 7):
        idx, _ = O.topk(s, k)
        sel = set(idx.tolist())
        assert len(sel) == k and all(0 <= t < 500 for t in sel)
        rest = np.array(sorted(set(range(500)) - sel), dtype=int)
        if len(rest):
            assert s[idx].min() >= s[rest].max()
        assert prev <= sel                                        # I_k subset of I_{k+7}
        prev = sel
    # among equal scores the lower index wins
    s = np.array([1.0, 5.0, 5.0, 0.0, 5.0])
    assert O.topk(s, 2)[0].tolist() == [1, 2]
    assert O.topk(s, 3)[0].tolist() == [1, 2, 4]
    assert O.topk(np.array([0.0, -0.0, -0.0, 0.0]), 2)[0].tolist() == [0, 1]


# ---------------------------------------------------------------- Algorithm 1, whole
@pytest.mark.parametrize("G", [1, 2])
def test_k_ge_L_equals_dense_for_any_channels(G):
    q, K, V = small_case(Hq=4 * G, Hkv=4, seed=20 + G)
    rng = np.random.default_rng(2)
    ch = np.stack([np.sort(rng.permutation(16)[:3]) for _ in range(4)]).astype(np.int32)
    lab = O.build_label(K, ch, 37)
    for k in (37, 50):
        out, idx = O.sparse_decode(q, lab, K, V, ch, 37, k)
        np.testing.assert_allclose(out, np_dense(q, K, V, 37), rtol=1e-12, atol=1e-13)
        assert (idx[..., :37] == np.arange(37)).all() and (idx[..., 37:] == -1).all()


def test_r_eq_d_identity_channels_k_eq_L_equals_dense():
    q, K, V = small_case(seed=31)
    ch = np.tile(np.arange(16, dtype=np.int32), (4, 1))
    lab = O.build_label(K, ch, 37)
    assert np.array_equal(lab.view(np.uint16), K.view(np.uint16))   # label == K
    out, _ = O.sparse_decode(q, lab, K, V, ch, 37, 37)
    np.testing.assert_allclose(out, O.dense_decode(q, K, V, 37), rtol=1e-12, atol=1e-13)
    # and with r = d the approximate score is the exact un-scaled logit
    s = O.scores(q, lab, ch, 37)
    want = np.einsum("bhd,bhtd->bht", q.astype(np.float64), K[:, :, :37].astype(np.float64))
    np.testing.assert_allclose(s, want, rtol=1e-13, atol=1e-13)


def test_sparse_equals_numpy_attention_over_bruteforce_selection():
    q, K, V = small_case(B=1, Hq=2, Hkv=2, d=16, L=60, L_max=64, seed=40)
    ch = np.array([[2, 3, 11], [0, 7, 9]], np.int32)
    lab = O.build_label(K, ch, 60)
    k = 9
    out, idx, sc, srt = O.sparse_decode(q, lab, K, V, ch, 60, k, want_scores=True)
    for h in range(2):
        s_hat = K[0, h, :60][:, ch[h]].astype(np.float64) @ q[0, h].astype(np.float64)[ch[h]]
        np.testing.assert_allclose(sc[0, h], s_hat, rtol=1e-13, atol=1e-13)
        I = brute_topk(sc[0, h].tolist(), k)
        assert idx[0, h].tolist() == I
        kk = K[0, h, I].astype(np.float64); vv = V[0, h, I].astype(np.float64)
        lg = kk @ q[0, h].astype(np.float64) / 4.0
        p = np.exp(lg - lg.max()); p /= p.sum()
        np.testing.assert_allclose(out[0, h], p @ vv, rtol=1e-12, atol=1e-13)
        assert np.array_equal(srt[0, h], np.sort(sc[0, h])[::-1])


def test_k1_returns_value_row_of_best_score_and_constant_rows():
    q, K, V = small_case(B=1, Hq=3, Hkv=3, d=16, L=33, L_max=33, seed=41)
    ch = np.array([[1, 2], [3, 4], [5, 6]], np.int32)
    lab = O.build_label(K, ch, 33)
    out, idx, sc, _ = O.sparse_decode(q, lab, K, V, ch, 33, 1, want_scores=True)
    for h in range(3):
        t = int(np.argmax(sc[0, h]))
        assert idx[0, h, 0] == t
        assert np.array_equal(out[0, h], V[0, h, t].astype(np.float64))
    # all V rows equal v -> y = v whatever is selected
    V2 = np.tile(V[:, :, :1], (1, 1, 33, 1))
    out2, _ = O.sparse_decode(q, lab, K, V2, ch, 33, 8)
    np.testing.assert_allclose(out2, V2[:, :, 0].astype(np.float64), rtol=1e-14, atol=1e-15)
    # y lies in the per-channel hull of the selected V rows; weights sum to 1
    out3, idx3 = O.sparse_decode(q, lab, K, V, ch, 33, 8)
    for h in range(3):
        rows = V[0, h, idx3[0, h]].astype(np.float64)
        assert (out3[0, h] <= rows.max(0) + 1e-12).all() and (out3[0, h] >= rows.min(0) - 1e-12).all()


def test_selection_invariant_to_power_of_two_query_scaling():
    q, K, V = small_case(B=1, Hq=2, Hkv=2, d=16, L=64, L_max=64, seed=42)
    ch = np.array([[0, 5, 6, 8], [1, 2, 3, 4]], np.int32)
    lab = O.build_label(K, ch, 64)
    _, idx = O.sparse_decode(q, lab, K, V, ch, 64, 10)
    q4 = (q.astype(np.float32) * 4).astype(np.float16)
    _, idx4 = O.sparse_decode(q4, lab, K, V, ch, 64, 10)
    assert np.array_equal(idx, idx4)
    # permuting the channel order (label columns follow) leaves integer-valued scores exact
    qi, Ki, Vi = small_case(B=1, Hq=2, Hkv=2, d=16, L=64, L_max=64, seed=43, ints=True)
    lab_a = O.build_label(Ki, ch, 64)
    chp = ch[:, ::-1].copy()
    lab_b = O.build_label(Ki, chp, 64)
    assert np.array_equal(O.scores(qi, lab_a, ch, 64), O.scores(qi, lab_b, chp, 64))


def test_gqa_group_of_identical_queries_selects_like_single_query():
    q1, K, V = small_case(B=2, Hq=2, Hkv=2, d=16, L=48, L_max=48, seed=44)
    G = 4
    qG = np.repeat(q1, G, axis=1)                                  # each KV head's group = G copies
    ch = np.array([[0, 3, 9], [4, 8, 12]], np.int32)
    lab = O.build_label(K, ch, 48)
    out1, idx1 = O.sparse_decode(q1, lab, K, V, ch, 48, 6)
    outG, idxG = O.sparse_decode(qG, lab, K, V, ch, 48, 6)
    assert np.array_equal(idx1, idxG)
    for g in range(G):
        np.testing.assert_allclose(outG[:, g::G], out1, rtol=1e-13, atol=1e-14)
    # group-summed scores: s_G = G * s_1 exactly (power of two)
    np.testing.assert_array_equal(O.scores(qG, lab, ch, 48), G * O.scores(q1, lab, ch, 48))


def test_gqa_heads_map_to_kv_head_hq_div_G():
    q, K, V = small_case(B=1, Hq=6, Hkv=2, d=16, L=20, L_max=20, seed=45)
    got = O.dense_decode(q, K, V, 20)
    for hq in range(6):
        one = O.dense_decode(q[:, hq:hq + 1], K[:, hq // 3:hq // 3 + 1], V[:, hq // 3:hq // 3 + 1], 20)
        np.testing.assert_array_equal(got[:, hq], one[:, 0])


def test_attend_idx_skips_negative_and_ignores_order():
    q, K, V = small_case(B=1, Hq=1, Hkv=1, d=16, L=30, L_max=30, seed=46)
    a = O.attend_idx(q, K, V, np.array([[[3, 9, 17, -1, -1]]], np.int32))
    b = O.attend_idx(q, K, V, np.array([[[17, -1, 3, 9, -1]]], np.int32))
    np.testing.assert_allclose(a, b, rtol=1e-14, atol=1e-15)
    I = [3, 9, 17]
    lg = K[0, 0, I].astype(np.float64) @ q[0, 0].astype(np.float64) / 4.0
    p = np.exp(lg - lg.max()); p /= p.sum()
    np.testing.assert_allclose(a[0, 0], p @ V[0, 0, I].astype(np.float64), rtol=1e-13)


# ---------------------------------------------------------------- calibration
@pytest.mark.parametrize("name", ["C1", "C4b"])
def test_calibration_recovers_seeded_outlier_channels(name):
    w = WORKLOADS[name]
    qc, kc = make_calibration_numpy(w, layer=3, N=512)
    want = outlier_channels(w.Hkv, w.d, layer=3)
    for mode in (0, 1, 2):
        ch, imp = O.calibrate(qc, kc, 8, mode)
        assert np.array_equal(ch, want)
    ch, _ = O.calibrate(qc, kc, w.d, 2)
    assert np.array_equal(ch, np.tile(np.arange(w.d), (w.Hkv, 1)))
    # r = 16 keeps the 8 outliers and adds 8 more
    ch16, _ = O.calibrate(qc, kc, 16, 2)
    for h in range(w.Hkv):
        assert set(want[h]) <= set(ch16[h]) and list(ch16[h]) == sorted(ch16[h])


def test_calibration_statistic_and_tie_rule():
    # N = 2, one KV head with G = 2 query heads, d = 4
    qc = np.array([[[1, -2, 0, 4], [3, 2, 0, 4]], [[-1, 2, 0, -4], [1, -2, 0, 4]]], np.float16)  # [N,Hq,d]
    kc = np.array([[[2, 1, 5, 1]], [[-2, 1, 5, 1]]], np.float16)                                  # [N,Hkv,d]
    _, imp_q = O.calibrate(qc, kc, 1, 0)
    _, imp_k = O.calibrate(qc, kc, 1, 1)
    _, imp_qk = O.calibrate(qc, kc, 1, 2)
    assert imp_q[0].tolist() == [1.5, 2.0, 0.0, 4.0]
    assert imp_k[0].tolist() == [2.0, 1.0, 5.0, 1.0]
    assert imp_qk[0].tolist() == [3.0, 2.0, 0.0, 4.0]
    assert O.calibrate(qc, kc, 2, 0)[0].tolist() == [[1, 3]]
    assert O.calibrate(qc, kc, 2, 1)[0].tolist() == [[0, 2]]
    assert O.calibrate(qc, kc, 2, 2)[0].tolist() == [[0, 3]]
    # equal importance keeps the lower channel: k-mode importances of channels 1 and 3 tie
    assert O.calibrate(qc, kc, 3, 1)[0].tolist() == [[0, 1, 2]]


# ---------------------------------------------------------------- workload recipe sanity
def test_workload_generator_is_seeded_and_has_static_outliers():
    w = WORKLOADS["C1"].scaled(L=256, k=16)
    a = make_layer_numpy(w, layer=0)
    b = make_layer_numpy(w, layer=0)
    assert all(np.array_equal(a[n].view(np.uint16), b[n].view(np.uint16)) for n in a)
    out = outlier_channels(w.Hkv, w.d, 0)
    K = a["K"].astype(np.float32)
    for h in range(0, w.Hkv, 7):
        std = K[0, h].std(0)
        assert (std[out[h]] > 6).all()
        rest = np.setdiff1d(np.arange(w.d), out[h])
        assert (std[rest] < 1.5).all()
    assert WORKLOADS["C3"].algorithmic_bytes() == 100663296
    assert WORKLOADS["C2"].algorithmic_bytes() == 268435456


def test_pins_hold_under_sanitizers():
    """The oracle built with -fsanitize=address,undefined passes every pin above in a process of
    its own (the ASan runtime has to be preloaded into the interpreter), and neither sanitizer
    reports anything: no read or write outside a buffer, no signed overflow, no misaligned access."""
    import subprocess
    import sys
    if O.SANITIZE:
        pytest.skip("already running on the sanitized build")
    O.build(sanitize=True)
    env = dict(os.environ)
    env["DS_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = ":".join(x for x in (O.asan_runtime(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-x", "-q", "-p", "no:cacheprovider"],
                         env=env, capture_output=True, text=True, timeout=900,
                         cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in res.stdout + res.stderr and "runtime error" not in res.stdout + res.stderr, tail
    assert " passed" in res.stdout, tail
