"""ctypes front end of the CPU oracle (``ds_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
bench's ``cpu_baseline`` leg, never by the product package.  Argument
marshalling only; all arithmetic is in the C file.  fp16 tensors are numpy
``float16`` arrays (viewed as uint16 bit patterns), results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ds_oracle.c")
_LIB = os.path.join(_HERE, "libds_oracle.so")
# The same source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).  A
# process that sets DS_ORACLE_SANITIZE=1 loads this build; it has to be started with the ASan
# runtime preloaded (see tests/test_oracle_pins.py::test_pins_hold_under_sanitizers).
_LIB_SAN = os.path.join(_HERE, "libds_oracle_san.so")
SANITIZE = os.environ.get("DS_ORACLE_SANITIZE", "") == "1"
_lib = None


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile ds_oracle.c with gcc (fp contraction off, OpenMP over units)."""
    lib = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
        cmd = ["gcc"] + opt + ["-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC",
                               "-shared", "-o", lib, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return lib


def asan_runtime() -> str:
    """Path of gcc's ASan runtime, to be preloaded by a process that loads the sanitized build."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build(sanitize=SANITIZE))
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError(f"{name} must be float16")
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def half_to_double(x):
    x = _u16(x, "x")
    out = np.empty(x.shape, dtype=np.float64)
    _load().ds_oracle_half_to_double(_p(x), _p(out), ctypes.c_int64(x.size))
    return out


def label_write(K, channels, label, t0, n):
    """In place: label[:, :, t0:t0+n, :] = K[:, :, t0:t0+n, channels] (Sec. 4.2)."""
    K = _u16(K, "K"); channels = _i32(channels)
    B, Hkv, L_max, d = K.shape
    r = channels.shape[1]
    assert label.dtype == np.float16 and label.flags.c_contiguous
    assert label.shape == (B, Hkv, L_max, r)
    assert 0 <= t0 and t0 + n <= L_max
    _load().ds_oracle_label_write(_p(K), _p(channels), _p(label), B, Hkv, L_max, d, r, t0, n)
    return label


def build_label(K, channels, L):
    B, Hkv, L_max, _ = K.shape
    label = np.zeros((B, Hkv, L_max, np.asarray(channels).shape[1]), dtype=np.float16)
    return label_write(K, channels, label, 0, L)


def append_kv(k_new, v_new, K, V, channels, label, t0):
    """Decode-step cache maintenance (Sec. 4.2): in place, the n new tokens' rows
    k_new, v_new [B,Hkv,n,d] become tokens [t0, t0+n) of K and V, and their
    channel values the same tokens of the label cache."""
    n = k_new.shape[2]
    assert t0 >= 0 and t0 + n <= K.shape[2]
    K[:, :, t0:t0 + n] = k_new
    V[:, :, t0:t0 + n] = v_new
    return label_write(K, channels, label, t0, n)


def predict_query(x, Wq):
    """Sec. 5.1: the approximate query of the next layer, its query projection applied
    to this layer's input embedding: q[b, n] = sum_m Wq[n, m] x[b, m], in float64,
    rounded once to fp16.  x [B, Dm], Wq [N, Dm] fp16 -> [B, N] fp16."""
    x = _u16(x, "x"); Wq = _u16(Wq, "Wq")
    return (x.astype(np.float64) @ Wq.astype(np.float64).T).astype(np.float16)


def interleave_kv(K, V):
    """[B,Hkv,L_max,2,d]: each token's K row followed by its V row."""
    return np.ascontiguousarray(np.stack([K, V], axis=3))


def label_q4_amax(K, channels, L):
    """4-bit label cache (Sec. 4.2), step 1: amax[B,Hkv,r] float32 over tokens [0, L)."""
    K = _u16(K, "K"); channels = _i32(channels)
    B, Hkv, L_max, d = K.shape
    r = channels.shape[1]
    amax = np.zeros((B, Hkv, r), dtype=np.float32)
    _load().ds_oracle_label_q4_amax(_p(K), _p(channels), _p(amax), B, Hkv, L, L_max, d, r)
    return amax


def label_q4_write(K, channels, amax, codes, t0, n):
    """In place: codes[:, :, t0:t0+n] = the packed 4-bit codes of K's label channels."""
    K = _u16(K, "K"); channels = _i32(channels)
    B, Hkv, L_max, d = K.shape
    r = channels.shape[1]
    assert codes.dtype == np.uint32 and codes.flags.c_contiguous and codes.shape == (B, Hkv, L_max, (r + 7) // 8)
    assert amax.dtype == np.float32 and amax.flags.c_contiguous and amax.shape == (B, Hkv, r)
    assert 0 <= t0 and t0 + n <= L_max
    _load().ds_oracle_label_q4_write(_p(K), _p(channels), _p(amax), _p(codes), B, Hkv, L_max, d, r, t0, n)
    return codes


def build_label_q4(K, channels, L):
    """(codes [B,Hkv,L_max,ceil(r/8)] uint32, amax [B,Hkv,r] float32)."""
    B, Hkv, L_max, _ = K.shape
    r = np.asarray(channels).shape[1]
    amax = label_q4_amax(K, channels, L)
    codes = np.zeros((B, Hkv, L_max, (r + 7) // 8), dtype=np.uint32)
    return label_q4_write(K, channels, amax, codes, 0, L), amax


def scores_q4(q, codes, amax, channels, L, precision=64):
    q = _u16(q, "q"); channels = _i32(channels)
    B, Hq, d = q.shape
    _, Hkv, L_max, _ = codes.shape
    r = channels.shape[1]
    out = np.empty((B, Hkv, L), dtype=np.float64)
    _load().ds_oracle_scores_q4(_p(q), _p(codes), _p(amax), _p(channels), _p(out),
                                B, Hq, Hkv, d, L, L_max, r, precision)
    return out


def sparse_decode_q4(q, codes, amax, K, V, channels, L, k, precision=64, want_scores=False):
    """Algorithm 1 with scores from the 4-bit label cache; returns like sparse_decode."""
    q = _u16(q, "q"); K = _u16(K, "K"); V = _u16(V, "V"); channels = _i32(channels)
    B, Hq, d = q.shape
    _, Hkv, L_max, _ = K.shape
    r = channels.shape[1]
    out = np.empty((B, Hq, d), dtype=np.float64)
    idx = np.empty((B, Hkv, k), dtype=np.int32)
    sc = np.empty((B, Hkv, L), dtype=np.float64) if want_scores else None
    srt = np.empty((B, Hkv, L), dtype=np.float64) if want_scores else None
    _load().ds_oracle_sparse_decode_q4(_p(q), _p(codes), _p(amax), _p(K), _p(V), _p(channels), _p(out), _p(idx),
                                       _p(sc) if want_scores else None, _p(srt) if want_scores else None,
                                       B, Hq, Hkv, d, L, L_max, r, k, precision)
    return (out, idx, sc, srt) if want_scores else (out, idx)


def scores(q, label, channels, L, precision=64):
    """Alg. 1 steps 1-2: [B,Hkv,L] float64 approximate scores."""
    q = _u16(q, "q"); label = _u16(label, "label"); channels = _i32(channels)
    B, Hq, d = q.shape
    _, Hkv, L_max, r = label.shape
    out = np.empty((B, Hkv, L), dtype=np.float64)
    _load().ds_oracle_scores(_p(q), _p(label), _p(channels), _p(out),
                             B, Hq, Hkv, d, L, L_max, r, precision)
    return out


def topk(s, k):
    """Alg. 1 step 3 on one score vector: (idx[k] ascending/-1 padded, sorted scores)."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    L = s.shape[0]
    idx = np.empty(k, dtype=np.int32)
    srt = np.empty(L, dtype=np.float64)
    _load().ds_oracle_topk(_p(s), L, k, _p(idx), _p(srt))
    return idx, srt


def attend_idx(q, K, V, idx):
    """Alg. 1 steps 4-5 over a given index list idx[B,Hkv,k] (-1 = skip)."""
    q = _u16(q, "q"); K = _u16(K, "K"); V = _u16(V, "V"); idx = _i32(idx)
    B, Hq, d = q.shape
    _, Hkv, L_max, _ = K.shape
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().ds_oracle_attend_idx(_p(q), _p(K), _p(V), _p(idx), _p(out),
                                 B, Hq, Hkv, d, L_max, idx.shape[2])
    return out


def dense_decode(q, K, V, L):
    """Sec. 2.1: softmax(q K^T / sqrt(d)) V over tokens [0, L)."""
    q = _u16(q, "q"); K = _u16(K, "K"); V = _u16(V, "V")
    B, Hq, d = q.shape
    _, Hkv, L_max, _ = K.shape
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().ds_oracle_dense_decode(_p(q), _p(K), _p(V), _p(out), B, Hq, Hkv, d, L, L_max)
    return out


def sparse_decode(q, label, K, V, channels, L, k, precision=64, want_scores=False):
    """Algorithm 1.  Returns (out[B,Hq,d] f64, idx[B,Hkv,k] i32) and, with
    want_scores, also (scores[B,Hkv,L], sorted_scores[B,Hkv,L] descending)."""
    q = _u16(q, "q"); label = _u16(label, "label"); K = _u16(K, "K"); V = _u16(V, "V")
    channels = _i32(channels)
    B, Hq, d = q.shape
    _, Hkv, L_max, r = label.shape
    out = np.empty((B, Hq, d), dtype=np.float64)
    idx = np.empty((B, Hkv, k), dtype=np.int32)
    sc = np.empty((B, Hkv, L), dtype=np.float64) if want_scores else None
    srt = np.empty((B, Hkv, L), dtype=np.float64) if want_scores else None
    _load().ds_oracle_sparse_decode(
        _p(q), _p(label), _p(K), _p(V), _p(channels), _p(out), _p(idx),
        _p(sc) if want_scores else None, _p(srt) if want_scores else None,
        B, Hq, Hkv, d, L, L_max, r, k, precision)
    if want_scores:
        return out, idx, sc, srt
    return out, idx


def calibrate(q_calib, k_calib, r, mode):
    """Sec. 4.1.  q_calib [N,Hq,d], k_calib [N,Hkv,d] fp16; mode 0=q, 1=k, 2=qk.
    Returns (channels[Hkv,r] ascending, importance[Hkv,d])."""
    q_calib = _u16(q_calib, "q_calib"); k_calib = _u16(k_calib, "k_calib")
    N, Hq, d = q_calib.shape
    Hkv = k_calib.shape[1]
    ch = np.empty((Hkv, r), dtype=np.int32)
    imp = np.empty((Hkv, d), dtype=np.float64)
    _load().ds_oracle_calibrate(_p(q_calib), _p(k_calib), N, Hq, Hkv, d, r, mode,
                                _p(ch), _p(imp))
    return ch, imp
