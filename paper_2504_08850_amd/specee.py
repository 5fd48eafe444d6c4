"""Python binding of libspecee.so (include/specee.h): argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch supplies device memory and
streams, nothing else); every computation happens inside the HIP library.  A
missing library is a hard error -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libspecee.so"
_lib = None

OP_PREDICT, OP_PREDICT_SWEEP, OP_PREDICT_TREE, OP_LM_HEAD, OP_VERIFY, OP_LAYER_LOOP, OP_VERIFY_Q4, \
    OP_PREDICT_TREE_Q4 = range(8)


class SpeceeError(RuntimeError):
    def __init__(self, fn, code):
        self.code = code
        msg = lib().specee_strerror(code).decode()
        super().__init__(f"{fn} failed: {msg} ({code})")


class Dims(C.Structure):
    _fields_ = [("d", C.c_int32), ("V", C.c_int32), ("K", C.c_int32), ("H", C.c_int32),
                ("eps", C.c_float), ("threshold", C.c_float)]


class Mlp(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p)]


class Sched(C.Structure):
    _fields_ = [("L", C.c_int32), ("Q", C.c_int32), ("radius", C.c_int32), ("filled", C.c_int32),
                ("head", C.c_int32), ("queue", C.c_int32 * 64), ("counter", C.c_int32 * 256)]


def lib():
    """Open the HIP library (built by paper_2504_08850_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_08850_amd.build` "
                "(there is no CPU or PyTorch fallback for the predictor)")
        _lib = C.CDLL(str(LIB_PATH))
        _lib.specee_strerror.restype = C.c_char_p
        _lib.specee_strerror.argtypes = [C.c_int]
        _lib.specee_workspace_bytes.restype = C.c_size_t
        _lib.specee_workspace_bytes.argtypes = [C.c_int, C.POINTER(Dims), C.c_int, C.c_int]
    return _lib


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(None)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _mlp(W1, w2, b1, b2):
    f16 = torch.float16
    return Mlp(_ptr(W1, f16).value, _ptr(b1, f16).value, _ptr(w2, f16).value, _ptr(b2, f16).value)


def _dims(d, V, K, H, eps, threshold):
    return Dims(int(d), int(V), int(K), int(H), float(eps), float(threshold))


def workspace_bytes(op, dims: Dims, n, Mcap=0) -> int:
    r = lib().specee_workspace_bytes(int(op), C.byref(dims), int(n), int(Mcap))
    if r == C.c_size_t(-1).value:
        raise SpeceeError("specee_workspace_bytes", -1)
    return int(r)


def _workspace(op, dims, n, Mcap, workspace, device):
    need = workspace_bytes(op, dims, n, Mcap)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    return workspace, C.c_size_t(workspace.numel() * workspace.element_size())


def predict(hidden, gamma, lm_head, ids, prev_probs, W1, w2, b1=None, b2=None, eps=1e-5, threshold=0.5,
            out=None, stream=None, done=None):
    """specee_predict: B tokens at one layer.  Returns dict(logits, probs, scores, exit).  `done` ([B] int32):
    tokens with a non-zero entry are skipped on the device."""
    B, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    H = w2.shape[0]
    dev = hidden.device
    if out is None:
        out = dict(logits=torch.empty((B, K), dtype=torch.float32, device=dev),
                   probs=torch.empty((B, K), dtype=torch.float32, device=dev),
                   scores=torch.empty((B,), dtype=torch.float32, device=dev),
                   exit=torch.empty((B,), dtype=torch.int32, device=dev))
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    f16 = torch.float16
    rc = lib().specee_predict(C.byref(dims), C.c_int(B), _ptr(hidden, f16), _ptr(gamma, f16), _ptr(lm_head, f16),
                              _ptr(ids, torch.int32), _ptr(prev_probs, torch.float32), C.byref(mlp),
                              _ptr(done, torch.int32), _ptr(out["logits"]), _ptr(out["probs"]), _ptr(out["scores"]), _ptr(out["exit"]),
                              _stream(stream))
    if rc:
        raise SpeceeError("specee_predict", rc)
    return out


def predict_q4(hidden, gamma, qweight, scales, zeros, group, ids, prev_probs, W1, w2, b1=None, b2=None, eps=1e-5,
               threshold=0.5, out=None, stream=None, done=None):
    """specee_predict_q4: specee_predict against a 4-bit group-quantised LM head (qweight int32/uint32 words
    [V][d/8], scales / zeros fp16 [V][d/group])."""
    B, d = hidden.shape
    V = qweight.shape[0]
    K = ids.shape[1]
    H = w2.shape[0]
    dev = hidden.device
    assert qweight.shape == (V, d // 8) and qweight.dtype == torch.int32, "codes travel as int32 words"
    assert scales.shape == (V, d // group) and zeros.shape == scales.shape
    if out is None:
        out = dict(logits=torch.empty((B, K), dtype=torch.float32, device=dev),
                   probs=torch.empty((B, K), dtype=torch.float32, device=dev),
                   scores=torch.empty((B,), dtype=torch.float32, device=dev),
                   exit=torch.empty((B,), dtype=torch.int32, device=dev))
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    f16 = torch.float16
    rc = lib().specee_predict_q4(C.byref(dims), C.c_int(B), _ptr(hidden, f16), _ptr(gamma, f16),
                                 _ptr(qweight, torch.int32), _ptr(scales, f16), _ptr(zeros, f16), C.c_int(group),
                                 _ptr(ids, torch.int32), _ptr(prev_probs, torch.float32), C.byref(mlp),
                                 _ptr(done, torch.int32), _ptr(out["logits"]), _ptr(out["probs"]),
                                 _ptr(out["scores"]), _ptr(out["exit"]), _stream(stream))
    if rc:
        raise SpeceeError("specee_predict_q4", rc)
    return out


def predict_sweep(hidden, gamma, lm_head, ids, W1, w2, b1=None, b2=None, prev0=None, active=None, eps=1e-5,
                  threshold=0.5, out=None, stream=None):
    """specee_predict_sweep: hidden [L][B][d], one predictor per layer."""
    L, B, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    H = w2.shape[1]
    dev = hidden.device
    if out is None:
        out = dict(logits=torch.empty((L, B, K), dtype=torch.float32, device=dev),
                   probs=torch.empty((L, B, K), dtype=torch.float32, device=dev),
                   scores=torch.empty((L, B), dtype=torch.float32, device=dev),
                   exit=torch.empty((L, B), dtype=torch.int32, device=dev),
                   first_exit=torch.empty((B,), dtype=torch.int32, device=dev))
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    f16 = torch.float16
    rc = lib().specee_predict_sweep(C.byref(dims), C.c_int(L), C.c_int(B), _ptr(hidden, f16), _ptr(gamma, f16),
                                    _ptr(lm_head, f16), _ptr(ids, torch.int32), _ptr(prev0, torch.float32),
                                    C.byref(mlp), _ptr(active, torch.int32), _ptr(out["logits"]),
                                    _ptr(out["probs"]), _ptr(out["scores"]), _ptr(out["exit"]),
                                    _ptr(out["first_exit"]), _stream(stream))
    if rc:
        raise SpeceeError("specee_predict_sweep", rc)
    return out


def layer_loop(hidden, gamma, lm_head, ids, W1, w2, b1=None, b2=None, prev0=None, active=None, eps=1e-5,
               threshold=0.5, spin_limit=0, out=None, workspace=None, stream=None):
    """specee_layer_loop: hidden [L][B][d], one predictor per layer; predict -> verify -> exit on the device."""
    L, B, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    H = w2.shape[1]
    dev = hidden.device
    if out is None:
        i32, f32 = torch.int32, torch.float32
        out = dict(logits=torch.empty((L, B, K), dtype=f32, device=dev), probs=torch.empty((L, B, K), dtype=f32, device=dev),
                   scores=torch.empty((L, B), dtype=f32, device=dev), exit=torch.empty((L, B), dtype=i32, device=dev),
                   ver_token=torch.empty((L, B), dtype=i32, device=dev), hit=torch.empty((L, B), dtype=i32, device=dev),
                   exit_layer=torch.empty((B,), dtype=i32, device=dev), token=torch.empty((B,), dtype=i32, device=dev),
                   status=torch.empty((B,), dtype=i32, device=dev))
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    workspace, wbytes = _workspace(OP_LAYER_LOOP, dims, B, 0, workspace, dev)
    f16 = torch.float16
    rc = lib().specee_layer_loop(C.byref(dims), C.c_int(L), C.c_int(B), _ptr(hidden, f16), _ptr(gamma, f16),
                                 _ptr(lm_head, f16), _ptr(ids, torch.int32), _ptr(prev0, torch.float32), C.byref(mlp),
                                 _ptr(active, torch.int32), _ptr(out["logits"]), _ptr(out["probs"]),
                                 _ptr(out["scores"]), _ptr(out["exit"]), _ptr(out["ver_token"]), _ptr(out["hit"]),
                                 _ptr(out["exit_layer"]), _ptr(out["token"]), _ptr(out["status"]),
                                 C.c_longlong(int(spin_limit)), _ptr(workspace), wbytes, _stream(stream))
    if rc:
        raise SpeceeError("specee_layer_loop", rc)
    out["_workspace"] = workspace
    return out


def layer_loop_q4(hidden, gamma, qweight, scales, zeros, group, ids, W1, w2, b1=None, b2=None, prev0=None, active=None,
                  eps=1e-5, threshold=0.5, spin_limit=0, out=None, workspace=None, stream=None):
    """specee_layer_loop_q4: layer_loop on the 4-bit group-quantised LM head (qweight int32/uint32 [V][d/8])."""
    L, B, d = hidden.shape
    V = qweight.shape[0]
    K = ids.shape[1]
    H = w2.shape[1]
    dev = hidden.device
    assert tuple(qweight.shape) == (V, d // 8) and tuple(scales.shape) == (V, d // group) == tuple(zeros.shape)
    if out is None:
        i32, f32 = torch.int32, torch.float32
        out = dict(logits=torch.empty((L, B, K), dtype=f32, device=dev), probs=torch.empty((L, B, K), dtype=f32, device=dev),
                   scores=torch.empty((L, B), dtype=f32, device=dev), exit=torch.empty((L, B), dtype=i32, device=dev),
                   ver_token=torch.empty((L, B), dtype=i32, device=dev), hit=torch.empty((L, B), dtype=i32, device=dev),
                   exit_layer=torch.empty((B,), dtype=i32, device=dev), token=torch.empty((B,), dtype=i32, device=dev),
                   status=torch.empty((B,), dtype=i32, device=dev))
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    workspace, wbytes = _workspace(OP_LAYER_LOOP, dims, B, 0, workspace, dev)
    f16 = torch.float16
    rc = lib().specee_layer_loop_q4(C.byref(dims), C.c_int(L), C.c_int(B), _ptr(hidden, f16), _ptr(gamma, f16),
                                    _ptr(qweight, torch.int32), _ptr(scales, f16), _ptr(zeros, f16), C.c_int(group),
                                    _ptr(ids, torch.int32), _ptr(prev0, torch.float32), C.byref(mlp),
                                    _ptr(active, torch.int32), _ptr(out["logits"]), _ptr(out["probs"]),
                                    _ptr(out["scores"]), _ptr(out["exit"]), _ptr(out["ver_token"]), _ptr(out["hit"]),
                                    _ptr(out["exit_layer"]), _ptr(out["token"]), _ptr(out["status"]),
                                    C.c_longlong(int(spin_limit)), _ptr(workspace), wbytes, _stream(stream))
    if rc:
        raise SpeceeError("specee_layer_loop_q4", rc)
    out["_workspace"] = workspace
    return out


def predict_tree(hidden, gamma, lm_head, ids, prev_probs, W1, w2, b1=None, b2=None, parent=None, Mcap=64,
                 eps=1e-5, threshold=0.5, want_path=None, out=None, workspace=None, stream=None):
    """specee_predict_tree: hidden [G][N][d] (or [N][d] for a single tree)."""
    single = hidden.dim() == 2
    if single:
        hidden, ids, prev_probs = hidden[None], ids[None], prev_probs[None]
        parent = None if parent is None else parent[None]
    G, N, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[2]
    H = w2.shape[0]
    dev = hidden.device
    if want_path is None:
        want_path = parent is not None
    if out is None:
        i32, f32 = torch.int32, torch.float32
        out = dict(merged=torch.empty((G, Mcap), dtype=i32, device=dev), M=torch.empty((G,), dtype=i32, device=dev),
                   cols=torch.empty((G, N, K), dtype=i32, device=dev),
                   logits=torch.empty((G, N, K), dtype=f32, device=dev),
                   probs=torch.empty((G, N, K), dtype=f32, device=dev),
                   scores=torch.empty((G, N), dtype=f32, device=dev),
                   exit=torch.empty((G, N), dtype=i32, device=dev),
                   path_exit=torch.empty((G, N), dtype=i32, device=dev) if want_path else None)
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    workspace, wbytes = _workspace(OP_PREDICT_TREE, dims, G * N, Mcap, workspace, dev)
    f16 = torch.float16
    rc = lib().specee_predict_tree(C.byref(dims), C.c_int(G), C.c_int(N), C.c_int(Mcap), _ptr(hidden, f16),
                                   _ptr(gamma, f16), _ptr(lm_head, f16), _ptr(ids, torch.int32),
                                   _ptr(parent, torch.int32), _ptr(prev_probs, torch.float32), C.byref(mlp),
                                   _ptr(out["merged"]), _ptr(out["M"]), _ptr(out["cols"]), _ptr(out["logits"]),
                                   _ptr(out["probs"]), _ptr(out["scores"]), _ptr(out["exit"]),
                                   _ptr(out.get("path_exit")), _ptr(workspace), wbytes, _stream(stream))
    if rc:
        raise SpeceeError("specee_predict_tree", rc)
    out["_workspace"] = workspace
    if single:
        return {k: (v[0] if (v is not None and k != "_workspace") else v) for k, v in out.items()}
    return out


def predict_tree_static(hidden, gamma, lm_head, ids, prev_probs, W1, w2, b1=None, b2=None, parent=None, Mcap=64,
                        eps=1e-5, threshold=0.5, out=None, stream=None):
    """specee_predict_tree_static: specee_predict_tree on the library's own static scratch array.  `out` must
    be given (dict with merged, M, cols, logits, probs, scores, exit and, with parent, path_exit): this binding
    allocates nothing either.  hidden [G][N][d]."""
    G, N, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[2]
    H = w2.shape[0]
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    f16 = torch.float16
    rc = lib().specee_predict_tree_static(C.byref(dims), C.c_int(G), C.c_int(N), C.c_int(Mcap), _ptr(hidden, f16),
                                          _ptr(gamma, f16), _ptr(lm_head, f16), _ptr(ids, torch.int32),
                                          _ptr(parent, torch.int32), _ptr(prev_probs, torch.float32), C.byref(mlp),
                                          _ptr(out["merged"]), _ptr(out["M"]), _ptr(out["cols"]),
                                          _ptr(out["logits"]), _ptr(out["probs"]), _ptr(out["scores"]),
                                          _ptr(out["exit"]), _ptr(out.get("path_exit")), _stream(stream))
    if rc:
        raise SpeceeError("specee_predict_tree_static", rc)
    return out


def lm_head_gemv(hidden, gamma, lm_head, eps=1e-5, out=None, workspace=None, stream=None):
    """lm_head_gemv: out [N][V] = RMSNorm(hidden) @ lm_head^T."""
    N, d = hidden.shape
    V = lm_head.shape[0]
    dev = hidden.device
    if out is None:
        out = torch.empty((N, V), dtype=torch.float32, device=dev)
    dims = _dims(d, V, 1, 1, eps, 0.5)
    workspace, wbytes = _workspace(OP_LM_HEAD, dims, N, 0, workspace, dev)
    f16 = torch.float16
    rc = lib().lm_head_gemv(C.byref(dims), C.c_int(N), _ptr(hidden, f16), _ptr(gamma, f16), _ptr(lm_head, f16),
                            _ptr(out, torch.float32), _ptr(workspace), wbytes, _stream(stream))
    if rc:
        raise SpeceeError("lm_head_gemv", rc)
    return out


def verify(hidden, gamma, lm_head, ids, gate=None, eps=1e-5, out=None, workspace=None, stream=None, done=None):
    """specee_verify: arg-max token of the full head and membership in the K ids; `gate` ([N] int32, e.g.
    the predictor's exit flags) skips hidden states whose entry is 0 on the device; `done` ([N] int32, in/out)
    skips states whose entry is non-zero and is set to 1 where the verification hits."""
    N, d = hidden.shape
    V = lm_head.shape[0]
    K = ids.shape[1]
    dev = hidden.device
    if out is None:
        out = dict(token=torch.empty((N,), dtype=torch.int32, device=dev),
                   max_logit=torch.empty((N,), dtype=torch.float32, device=dev),
                   hit=torch.empty((N,), dtype=torch.int32, device=dev))
    dims = _dims(d, V, K, 1, eps, 0.5)
    workspace, wbytes = _workspace(OP_VERIFY, dims, N, 0, workspace, dev)
    f16 = torch.float16
    rc = lib().specee_verify(C.byref(dims), C.c_int(N), _ptr(hidden, f16), _ptr(gamma, f16), _ptr(lm_head, f16),
                             _ptr(ids, torch.int32), _ptr(gate, torch.int32), _ptr(done, torch.int32),
                             _ptr(out["token"]),
                             _ptr(out["max_logit"]), _ptr(out["hit"]),
                             _ptr(workspace), wbytes, _stream(stream))
    if rc:
        raise SpeceeError("specee_verify", rc)
    return out


def _q4_args(qweight, scales, zeros, group, d):
    V = qweight.shape[0]
    assert qweight.shape == (V, d // 8) and qweight.dtype == torch.int32, "codes travel as int32 words"
    assert scales.shape == (V, d // group) and zeros.shape == scales.shape
    f16 = torch.float16
    return V, (_ptr(qweight, torch.int32), _ptr(scales, f16), _ptr(zeros, f16), C.c_int(group))


def lm_head_gemv_q4(hidden, gamma, qweight, scales, zeros, group, eps=1e-5, out=None, stream=None):
    """lm_head_gemv_q4: out [N][V] against the 4-bit group-quantised head."""
    N, d = hidden.shape
    V, q = _q4_args(qweight, scales, zeros, group, d)
    if out is None:
        out = torch.empty((N, V), dtype=torch.float32, device=hidden.device)
    dims = _dims(d, V, 1, 1, eps, 0.5)
    f16 = torch.float16
    rc = lib().lm_head_gemv_q4(C.byref(dims), C.c_int(N), _ptr(hidden, f16), _ptr(gamma, f16), *q,
                               _ptr(out, torch.float32), _stream(stream))
    if rc:
        raise SpeceeError("lm_head_gemv_q4", rc)
    return out


def verify_q4(hidden, gamma, qweight, scales, zeros, group, ids, gate=None, eps=1e-5, out=None, workspace=None,
              stream=None, done=None):
    """specee_verify_q4: specee_verify against the 4-bit group-quantised head."""
    N, d = hidden.shape
    V, q = _q4_args(qweight, scales, zeros, group, d)
    K = ids.shape[1]
    dev = hidden.device
    if out is None:
        out = dict(token=torch.empty((N,), dtype=torch.int32, device=dev),
                   max_logit=torch.empty((N,), dtype=torch.float32, device=dev),
                   hit=torch.empty((N,), dtype=torch.int32, device=dev))
    dims = _dims(d, V, K, 1, eps, 0.5)
    workspace, wbytes = _workspace(OP_VERIFY_Q4, dims, N, 0, workspace, dev)
    f16 = torch.float16
    rc = lib().specee_verify_q4(C.byref(dims), C.c_int(N), _ptr(hidden, f16), _ptr(gamma, f16), *q,
                                _ptr(ids, torch.int32), _ptr(gate, torch.int32), _ptr(done, torch.int32),
                                _ptr(out["token"]), _ptr(out["max_logit"]), _ptr(out["hit"]), _ptr(workspace), wbytes,
                                _stream(stream))
    if rc:
        raise SpeceeError("specee_verify_q4", rc)
    return out


def predict_tree_q4(hidden, gamma, qweight, scales, zeros, group, ids, prev_probs, W1, w2, b1=None, b2=None,
                    parent=None, Mcap=64, eps=1e-5, threshold=0.5, out=None, stream=None):
    """specee_predict_tree_q4: hidden [G][N][d] (or [N][d] for a single tree) against the quantised head."""
    single = hidden.dim() == 2
    if single:
        hidden, ids, prev_probs = hidden[None], ids[None], prev_probs[None]
        parent = None if parent is None else parent[None]
    G, N, d = hidden.shape
    V, q = _q4_args(qweight, scales, zeros, group, d)
    K = ids.shape[2]
    H = w2.shape[0]
    dev = hidden.device
    if out is None:
        i32, f32 = torch.int32, torch.float32
        out = dict(merged=torch.empty((G, Mcap), dtype=i32, device=dev), M=torch.empty((G,), dtype=i32, device=dev),
                   cols=torch.empty((G, N, K), dtype=i32, device=dev),
                   logits=torch.empty((G, N, K), dtype=f32, device=dev),
                   probs=torch.empty((G, N, K), dtype=f32, device=dev),
                   scores=torch.empty((G, N), dtype=f32, device=dev),
                   exit=torch.empty((G, N), dtype=i32, device=dev),
                   path_exit=torch.empty((G, N), dtype=i32, device=dev) if parent is not None else None)
    dims = _dims(d, V, K, H, eps, threshold)
    mlp = _mlp(W1, w2, b1, b2)
    f16 = torch.float16
    rc = lib().specee_predict_tree_q4(C.byref(dims), C.c_int(G), C.c_int(N), C.c_int(Mcap), _ptr(hidden, f16),
                                      _ptr(gamma, f16), *q, _ptr(ids, torch.int32), _ptr(parent, torch.int32),
                                      _ptr(prev_probs, torch.float32), C.byref(mlp), _ptr(out["merged"]),
                                      _ptr(out["M"]), _ptr(out["cols"]), _ptr(out["logits"]), _ptr(out["probs"]),
                                      _ptr(out["scores"]), _ptr(out["exit"]), _ptr(out.get("path_exit")),
                                      _stream(stream))
    if rc:
        raise SpeceeError("specee_predict_tree_q4", rc)
    if single:
        return {k: (v[0] if v is not None else None) for k, v in out.items()}
    return out


def status_word(scores, M=None, Mcap=0, out=None, stream=None):
    """specee_status_word: one int32 on the device (bit 1: an invalid id somewhere, bit 2: a merged set overflowed)."""
    if out is None:
        out = torch.empty((1,), dtype=torch.int32, device=scores.device)
    G = 0 if M is None else M.numel()
    rc = lib().specee_status_word(_ptr(scores, torch.float32), C.c_size_t(scores.numel()), _ptr(M, torch.int32),
                                  C.c_int(G), C.c_int(Mcap), _ptr(out, torch.int32), _stream(stream))
    if rc:
        raise SpeceeError("specee_status_word", rc)
    return out


def calib_copy(dst, src, stream=None):
    """specee_calib_copy: plain device copy of known size (counter calibration)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    rc = lib().specee_calib_copy(_ptr(dst), _ptr(src), C.c_size_t(nbytes), _stream(stream))
    if rc:
        raise SpeceeError("specee_calib_copy", rc)
    return dst


class Scheduler:
    """Host-side online scheduler (specee_sched_*): circular queue of recent exit layers."""

    def __init__(self, L, Q=5, radius=2, offline_mask=None):
        self._s = Sched()
        rc = lib().specee_sched_init(C.byref(self._s), int(L), int(Q), int(radius))
        if rc:
            raise SpeceeError("specee_sched_init", rc)
        self.L = L
        self._mask = None
        if offline_mask is not None:
            self._mask = (C.c_int32 * L)(*[int(x) for x in offline_mask])
        self._active = (C.c_int32 * L)()

    def push(self, exit_layer):
        rc = lib().specee_sched_push(C.byref(self._s), int(exit_layer))
        if rc:
            raise SpeceeError("specee_sched_push", rc)

    def active(self):
        n = lib().specee_sched_active(C.byref(self._s), self._mask, self._active)
        if n < 0:
            raise SpeceeError("specee_sched_active", n)
        return list(self._active)

    def counters(self):
        return list(self._s.counter[: self.L])
