"""ctypes front end of the CPU oracle (oracle/specee_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module,
and this module never imports the product package.

Arrays go in as numpy (float16 for half-precision tensors, int32, float32) and
come back as float64 / int32.  The C file holds all the arithmetic; this file
only marshals arguments and compiles the C with gcc on first use.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "specee_ref.c"
_LIB = _HERE / "libspecee_ref.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (plain -O2, OpenMP for the outer loops)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-ffp-contract=off", str(_SRC), "-o", str(tmp), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _p(a, t):
    return None if a is None else a.ctypes.data_as(C.POINTER(t))


def _h(a):
    """float16 array -> contiguous uint16 view."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a.view(np.uint16)


def _i(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _f(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(str(build()))
        _lib.specee_ref_half_to_double.restype = C.c_double
        _lib.specee_ref_half_to_double.argtypes = [C.c_uint16]
        _lib.specee_ref_rms_scale.restype = C.c_double
        _lib.specee_ref_rms_scale.argtypes = [C.POINTER(C.c_uint16), C.c_int, C.c_double]
    return _lib


def set_threads(n: int) -> None:
    lib().specee_ref_set_threads(C.c_int(int(n)))


def get_threads() -> int:
    return int(lib().specee_ref_get_threads())


def half_to_double(bits: int) -> float:
    return float(lib().specee_ref_half_to_double(C.c_uint16(int(bits))))


def rms_scale(h, eps: float) -> float:
    h = _h(h)
    return float(lib().specee_ref_rms_scale(_p(h, C.c_uint16), C.c_int(h.size), C.c_double(eps)))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def predict(hidden, gamma, lm_head, ids, prev_probs, W1, w2, b1=None, b2=None, eps=1e-5, threshold=0.5):
    """B tokens at one layer.  Returns dict(logits, probs, features, scores, exit)."""
    hidden, gamma, lm_head = _h(hidden), _h(gamma), _h(lm_head)
    ids, prev = _i(ids), _f(prev_probs)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    B, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    H = w2.shape[0]
    assert lm_head.shape[1] == d and gamma.shape == (d,) and ids.shape == (B, K) and prev.shape == (B, K)
    assert W1.shape == (H, 3 * K)
    logits = np.zeros((B, K)); probs = np.zeros((B, K)); feats = np.zeros((B, 3 * K))
    scores = np.zeros(B); ex = np.zeros(B, dtype=np.int32)
    u16, i32, f32, f64 = C.c_uint16, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_predict_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold), C.c_int(B),
        _p(hidden, u16), _p(gamma, u16), _p(lm_head, u16), _p(ids, i32), _p(prev, f32),
        _p(W1, u16), _p(b1, u16), _p(w2, u16), _p(b2, u16),
        _p(logits, f64), _p(probs, f64), _p(feats, f64), _p(scores, f64), _p(ex, i32))
    _check(rc, "specee_predict_ref")
    return dict(logits=logits, probs=probs, features=feats, scores=scores, exit=ex)


def predict_q4(hidden, gamma, qweight, scales, zeros, group, ids, prev_probs, W1, w2, b1=None, b2=None, eps=1e-5,
               threshold=0.5):
    """specee_predict_q4_ref: the predictor against a 4-bit group-quantised LM head
    (qweight uint32 [V][d/8], scales / zeros fp16 [V][d/group])."""
    hidden, gamma, scales, zeros = _h(hidden), _h(gamma), _h(scales), _h(zeros)
    qweight = np.ascontiguousarray(qweight, dtype=np.uint32)
    ids, prev = _i(ids), _f(prev_probs)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    B, d = hidden.shape
    V = qweight.shape[0]
    K = ids.shape[1]
    H = w2.shape[0]
    assert qweight.shape == (V, d // 8) and scales.shape == (V, d // group) and zeros.shape == scales.shape
    assert W1.shape == (H, 3 * K) and ids.shape == (B, K) and prev.shape == (B, K)
    logits = np.zeros((B, K)); probs = np.zeros((B, K)); feats = np.zeros((B, 3 * K))
    scores = np.zeros(B); ex = np.zeros(B, dtype=np.int32)
    u16, u32, i32, f32, f64 = C.c_uint16, C.c_uint32, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_predict_q4_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold), C.c_int(B),
        _p(hidden, u16), _p(gamma, u16), _p(qweight, u32), _p(scales, u16), _p(zeros, u16), C.c_int(group),
        _p(ids, i32), _p(prev, f32), _p(W1, u16), _p(b1, u16), _p(w2, u16), _p(b2, u16),
        _p(logits, f64), _p(probs, f64), _p(feats, f64), _p(scores, f64), _p(ex, i32))
    _check(rc, "specee_predict_q4_ref")
    return dict(logits=logits, probs=probs, features=feats, scores=scores, exit=ex)


def predict_sweep(hidden, gamma, lm_head, ids, W1, w2, b1=None, b2=None, prev0=None, active=None,
                  eps=1e-5, threshold=0.5):
    """L layers x B tokens with the probabilities carried layer to layer.
    hidden [L][B][d]; W1 [L][H][3K]; w2 [L][H]; b1 [L][H] / b2 [L] optional."""
    hidden, gamma, lm_head = _h(hidden), _h(gamma), _h(lm_head)
    ids, prev0, active = _i(ids), _f(prev0), _i(active)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    L, B, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    H = w2.shape[1]
    assert W1.shape == (L, H, 3 * K) and w2.shape == (L, H) and ids.shape == (B, K)
    logits = np.zeros((L, B, K)); probs = np.zeros((L, B, K)); scores = np.zeros((L, B))
    ex = np.zeros((L, B), dtype=np.int32); first = np.zeros(B, dtype=np.int32)
    u16, i32, f32, f64 = C.c_uint16, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_predict_sweep_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold),
        C.c_int(L), C.c_int(B), _p(hidden, u16), _p(gamma, u16), _p(lm_head, u16), _p(ids, i32),
        _p(prev0, f32), _p(W1, u16), _p(b1, u16), _p(w2, u16), _p(b2, u16), _p(active, i32),
        _p(logits, f64), _p(probs, f64), _p(scores, f64), _p(ex, i32), _p(first, i32))
    _check(rc, "specee_predict_sweep_ref")
    return dict(logits=logits, probs=probs, scores=scores, exit=ex, first_exit=first)


def merge(ids, cap: int):
    """Sorted distinct ids (padded with -1 to cap), their count, and the column of every id."""
    ids = _i(ids)
    merged = np.zeros(cap, dtype=np.int32); M = np.zeros(1, dtype=np.int32)
    cols = np.zeros(ids.shape, dtype=np.int32)
    rc = lib().specee_merge_ref(_p(ids, C.c_int32), C.c_int(ids.size), _p(merged, C.c_int32), C.c_int(cap),
                                _p(M, C.c_int32), _p(cols, C.c_int32))
    _check(rc, "specee_merge_ref")
    return merged, int(M[0]), cols


def predict_tree(hidden, gamma, lm_head, ids, prev_probs, W1, w2, b1=None, b2=None, parent=None, Mcap=64,
                 eps=1e-5, threshold=0.5, want_path=None):
    """G trees of N nodes.  hidden [G][N][d] (or [N][d] for one tree); ids [G][N][K]."""
    single = hidden.ndim == 2
    if single:
        hidden, ids, prev_probs = hidden[None], np.asarray(ids)[None], np.asarray(prev_probs)[None]
        parent = None if parent is None else np.asarray(parent)[None]
    hidden, gamma, lm_head = _h(hidden), _h(gamma), _h(lm_head)
    ids, prev, parent = _i(ids), _f(prev_probs), _i(parent)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    G, N, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[2]
    H = w2.shape[0]
    assert ids.shape == (G, N, K) and prev.shape == (G, N, K) and W1.shape == (H, 3 * K)
    if want_path is None:
        want_path = parent is not None
    merged = np.zeros((G, Mcap), dtype=np.int32); M = np.zeros(G, dtype=np.int32)
    cols = np.zeros((G, N, K), dtype=np.int32); Z = np.zeros((G, N, Mcap))
    logits = np.zeros((G, N, K)); probs = np.zeros((G, N, K)); scores = np.zeros((G, N))
    ex = np.zeros((G, N), dtype=np.int32)
    path = np.zeros((G, N), dtype=np.int32) if want_path else None
    u16, i32, f32, f64 = C.c_uint16, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_predict_tree_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold),
        C.c_int(G), C.c_int(N), C.c_int(Mcap), _p(hidden, u16), _p(gamma, u16), _p(lm_head, u16),
        _p(ids, i32), _p(parent, i32), _p(prev, f32), _p(W1, u16), _p(b1, u16), _p(w2, u16), _p(b2, u16),
        _p(merged, i32), _p(M, i32), _p(cols, i32), _p(Z, f64), _p(logits, f64), _p(probs, f64),
        _p(scores, f64), _p(ex, i32), _p(path, i32))
    _check(rc, "specee_predict_tree_ref")
    out = dict(merged=merged, M=M, cols=cols, Z=Z, logits=logits, probs=probs, scores=scores, exit=ex,
               path_exit=path)
    if single:
        out = {k: (v[0] if v is not None else None) for k, v in out.items()}
    return out


def lm_head_gemv(hidden, gamma, lm_head, eps=1e-5):
    hidden, gamma, lm_head = _h(hidden), _h(gamma), _h(lm_head)
    N, d = hidden.shape
    V = lm_head.shape[0]
    out = np.zeros((N, V))
    rc = lib().lm_head_gemv_ref(C.c_int(d), C.c_int(V), C.c_double(eps), C.c_int(N), _p(hidden, C.c_uint16),
                                _p(gamma, C.c_uint16), _p(lm_head, C.c_uint16), _p(out, C.c_double))
    _check(rc, "lm_head_gemv_ref")
    return out


def lm_head_rows(hidden, gamma, lm_head, rows, eps=1e-5):
    hidden, gamma, lm_head, rows = _h(hidden), _h(gamma), _h(lm_head), _i(rows)
    N, d = hidden.shape
    V = lm_head.shape[0]
    out = np.zeros((N, rows.size))
    rc = lib().lm_head_rows_ref(C.c_int(d), C.c_int(V), C.c_double(eps), C.c_int(N), _p(hidden, C.c_uint16),
                                _p(gamma, C.c_uint16), _p(lm_head, C.c_uint16), _p(rows, C.c_int32),
                                C.c_int(rows.size), _p(out, C.c_double))
    _check(rc, "lm_head_rows_ref")
    return out


def verify(hidden, gamma, lm_head, ids, eps=1e-5):
    hidden, gamma, lm_head, ids = _h(hidden), _h(gamma), _h(lm_head), _i(ids)
    N, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    token = np.zeros(N, dtype=np.int32); mx = np.zeros(N); hit = np.zeros(N, dtype=np.int32)
    rc = lib().specee_verify_ref(C.c_int(d), C.c_int(V), C.c_int(K), C.c_double(eps), C.c_int(N),
                                 _p(hidden, C.c_uint16), _p(gamma, C.c_uint16), _p(lm_head, C.c_uint16),
                                 _p(ids, C.c_int32), _p(token, C.c_int32), _p(mx, C.c_double), _p(hit, C.c_int32))
    _check(rc, "specee_verify_ref")
    return dict(token=token, max_logit=mx, hit=hit)


def _q4(qweight, scales, zeros, group, d):
    qweight = np.ascontiguousarray(qweight, dtype=np.uint32)
    scales, zeros = _h(scales), _h(zeros)
    V = qweight.shape[0]
    assert qweight.shape == (V, d // 8) and scales.shape == (V, d // group) and zeros.shape == scales.shape
    return qweight, scales, zeros, V


def lm_head_gemv_q4(hidden, gamma, qweight, scales, zeros, group, eps=1e-5):
    """Every vocabulary logit against the 4-bit group-quantised head: out [N][V]."""
    hidden, gamma = _h(hidden), _h(gamma)
    N, d = hidden.shape
    qweight, scales, zeros, V = _q4(qweight, scales, zeros, group, d)
    out = np.zeros((N, V))
    u16 = C.c_uint16
    rc = lib().lm_head_gemv_q4_ref(C.c_int(d), C.c_int(V), C.c_double(eps), C.c_int(N), _p(hidden, u16),
                                   _p(gamma, u16), _p(qweight, C.c_uint32), _p(scales, u16), _p(zeros, u16),
                                   C.c_int(group), _p(out, C.c_double))
    _check(rc, "lm_head_gemv_q4_ref")
    return out


def verify_q4(hidden, gamma, qweight, scales, zeros, group, ids, eps=1e-5):
    hidden, gamma, ids = _h(hidden), _h(gamma), _i(ids)
    N, d = hidden.shape
    qweight, scales, zeros, V = _q4(qweight, scales, zeros, group, d)
    K = ids.shape[1]
    token = np.zeros(N, dtype=np.int32); mx = np.zeros(N); hit = np.zeros(N, dtype=np.int32)
    u16 = C.c_uint16
    rc = lib().specee_verify_q4_ref(C.c_int(d), C.c_int(V), C.c_int(K), C.c_double(eps), C.c_int(N),
                                    _p(hidden, u16), _p(gamma, u16), _p(qweight, C.c_uint32), _p(scales, u16),
                                    _p(zeros, u16), C.c_int(group), _p(ids, C.c_int32), _p(token, C.c_int32),
                                    _p(mx, C.c_double), _p(hit, C.c_int32))
    _check(rc, "specee_verify_q4_ref")
    return dict(token=token, max_logit=mx, hit=hit)


def predict_tree_q4(hidden, gamma, qweight, scales, zeros, group, ids, prev_probs, W1, w2, b1=None, b2=None,
                    parent=None, Mcap=64, eps=1e-5, threshold=0.5):
    """G trees of N nodes against the quantised head.  hidden [G][N][d] (or [N][d]); ids [G][N][K]."""
    single = hidden.ndim == 2
    if single:
        hidden, ids, prev_probs = hidden[None], np.asarray(ids)[None], np.asarray(prev_probs)[None]
        parent = None if parent is None else np.asarray(parent)[None]
    hidden, gamma = _h(hidden), _h(gamma)
    ids, prev, parent = _i(ids), _f(prev_probs), _i(parent)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    G, N, d = hidden.shape
    qweight, scales, zeros, V = _q4(qweight, scales, zeros, group, d)
    K = ids.shape[2]
    H = w2.shape[0]
    assert ids.shape == (G, N, K) and prev.shape == (G, N, K) and W1.shape == (H, 3 * K)
    merged = np.zeros((G, Mcap), dtype=np.int32); M = np.zeros(G, dtype=np.int32)
    cols = np.zeros((G, N, K), dtype=np.int32)
    logits = np.zeros((G, N, K)); probs = np.zeros((G, N, K)); scores = np.zeros((G, N))
    ex = np.zeros((G, N), dtype=np.int32)
    path = np.zeros((G, N), dtype=np.int32) if parent is not None else None
    u16, u32, i32, f32, f64 = C.c_uint16, C.c_uint32, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_predict_tree_q4_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold),
        C.c_int(G), C.c_int(N), C.c_int(Mcap), _p(hidden, u16), _p(gamma, u16), _p(qweight, u32), _p(scales, u16),
        _p(zeros, u16), C.c_int(group), _p(ids, i32), _p(parent, i32), _p(prev, f32), _p(W1, u16), _p(b1, u16),
        _p(w2, u16), _p(b2, u16), _p(merged, i32), _p(M, i32), _p(cols, i32), _p(logits, f64), _p(probs, f64),
        _p(scores, f64), _p(ex, i32), _p(path, i32))
    _check(rc, "specee_predict_tree_q4_ref")
    out = dict(merged=merged, M=M, cols=cols, logits=logits, probs=probs, scores=scores, exit=ex, path_exit=path)
    if single:
        out = {k: (v[0] if v is not None else None) for k, v in out.items()}
    return out


def layer_loop(hidden, gamma, lm_head, ids, W1, w2, b1=None, b2=None, prev0=None, active=None, eps=1e-5,
               threshold=0.5):
    """The early-exit loop of B tokens down L layers: predictor at every active layer, verification after a
    positive prediction, exit at the first accepted verification.  hidden [L][B][d]; one predictor per layer."""
    hidden, gamma, lm_head = _h(hidden), _h(gamma), _h(lm_head)
    ids, prev0, active = _i(ids), _f(prev0), _i(active)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    L, B, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    H = w2.shape[1]
    assert W1.shape == (L, H, 3 * K) and w2.shape == (L, H) and ids.shape == (B, K)
    logits = np.zeros((L, B, K)); probs = np.zeros((L, B, K)); scores = np.zeros((L, B))
    ex = np.zeros((L, B), dtype=np.int32); vt = np.zeros((L, B), dtype=np.int32); hit = np.zeros((L, B), dtype=np.int32)
    exit_layer = np.zeros(B, dtype=np.int32); token = np.zeros(B, dtype=np.int32)
    u16, i32, f32, f64 = C.c_uint16, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_layer_loop_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold),
        C.c_int(L), C.c_int(B), _p(hidden, u16), _p(gamma, u16), _p(lm_head, u16), _p(ids, i32),
        _p(prev0, f32), _p(W1, u16), _p(b1, u16), _p(w2, u16), _p(b2, u16), _p(active, i32),
        _p(logits, f64), _p(probs, f64), _p(scores, f64), _p(ex, i32), _p(vt, i32), _p(hit, i32),
        _p(exit_layer, i32), _p(token, i32))
    _check(rc, "specee_layer_loop_ref")
    return dict(logits=logits, probs=probs, scores=scores, exit=ex, ver_token=vt, hit=hit, exit_layer=exit_layer,
                token=token)


def layer_loop_q4(hidden, gamma, qweight, scales, zeros, group, ids, W1, w2, b1=None, b2=None, prev0=None, active=None,
                  eps=1e-5, threshold=0.5):
    """layer_loop on the 4-bit group-quantised LM head (format of predict_q4)."""
    hidden, gamma = _h(hidden), _h(gamma)
    qweight = np.ascontiguousarray(qweight).view(np.uint32)
    scales, zeros = _h(scales), _h(zeros)
    ids, prev0, active = _i(ids), _f(prev0), _i(active)
    W1, w2, b1, b2 = _h(W1), _h(w2), _h(b1), _h(b2)
    L, B, d = hidden.shape
    V = qweight.shape[0]
    K = ids.shape[1]
    H = w2.shape[1]
    assert qweight.shape == (V, d // 8) and scales.shape == (V, d // group) and zeros.shape == scales.shape
    assert W1.shape == (L, H, 3 * K) and w2.shape == (L, H) and ids.shape == (B, K)
    logits = np.zeros((L, B, K)); probs = np.zeros((L, B, K)); scores = np.zeros((L, B))
    ex = np.zeros((L, B), dtype=np.int32); vt = np.zeros((L, B), dtype=np.int32); hit = np.zeros((L, B), dtype=np.int32)
    exit_layer = np.zeros(B, dtype=np.int32); token = np.zeros(B, dtype=np.int32)
    u16, u32, i32, f32, f64 = C.c_uint16, C.c_uint32, C.c_int32, C.c_float, C.c_double
    rc = lib().specee_layer_loop_q4_ref(
        C.c_int(d), C.c_int(V), C.c_int(K), C.c_int(H), C.c_double(eps), C.c_float(threshold),
        C.c_int(L), C.c_int(B), _p(hidden, u16), _p(gamma, u16), _p(qweight, u32), _p(scales, u16), _p(zeros, u16),
        C.c_int(group), _p(ids, i32), _p(prev0, f32), _p(W1, u16), _p(b1, u16), _p(w2, u16), _p(b2, u16),
        _p(active, i32), _p(logits, f64), _p(probs, f64), _p(scores, f64), _p(ex, i32), _p(vt, i32), _p(hit, i32),
        _p(exit_layer, i32), _p(token, i32))
    _check(rc, "specee_layer_loop_q4_ref")
    return dict(logits=logits, probs=probs, scores=scores, exit=ex, ver_token=vt, hit=hit, exit_layer=exit_layer,
                token=token)


def schedule(exit_layers, L: int, Q: int = 5, radius: int = 2, offline_mask=None):
    exit_layers, offline_mask = _i(exit_layers), _i(offline_mask)
    T = exit_layers.size
    active = np.zeros((T, L), dtype=np.int32); counters = np.zeros((T, L), dtype=np.int32)
    rc = lib().specee_schedule_ref(C.c_int(L), C.c_int(Q), C.c_int(radius), C.c_int(T),
                                   _p(exit_layers, C.c_int32), _p(offline_mask, C.c_int32),
                                   _p(active, C.c_int32), _p(counters, C.c_int32))
    _check(rc, "specee_schedule_ref")
    return active, counters
