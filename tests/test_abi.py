"""CPU-only checks of the boundary: the built library exports every function the public header
declares, host-side argument validation works without a GPU (no pointer is dereferenced before
validation fails), and the host-side scheduler matches the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "specee.h")


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    if not specee.LIB_PATH.exists():
        from paper_2504_08850_amd import build
        build.build(verbose=False)
    specee.lib()
    return specee


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^(?:int|size_t|const char \*)\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("specee_predict", "specee_predict_tree", "lm_head_gemv", "specee_predict_sweep", "specee_verify",
                 "specee_layer_loop", "specee_predict_q4", "lm_head_gemv_q4", "specee_verify_q4",
                 "specee_predict_tree_q4", "specee_layer_loop_q4", "specee_predict_tree_static", "specee_status_word",
                 "specee_workspace_bytes", "specee_strerror", "specee_version"):
        assert must in names


def test_library_exports_every_declared_symbol(sp):
    lib = sp.lib()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in specee.h but not exported"


def test_missing_library_is_a_hard_error(sp, monkeypatch, tmp_path):
    monkeypatch.setattr(sp, "_lib", None)
    monkeypatch.setattr(sp, "LIB_PATH", tmp_path / "libspecee.so")
    with pytest.raises(FileNotFoundError):
        sp.lib()


def test_version_and_strerror(sp):
    lib = sp.lib()
    assert lib.specee_version() >= 100
    assert lib.specee_strerror(0) == b"success"
    for code in (-1, -2, -3, -4, -5):
        assert lib.specee_strerror(code) not in (b"success", b"unknown status")
    assert lib.specee_strerror(-99) == b"unknown status"


def test_host_side_validation_without_a_gpu(sp):
    lib = sp.lib()
    fake = C.c_void_p(0x1000)       # aligned, never dereferenced: validation fails first
    odd = C.c_void_p(0x1008)
    mlp = sp.Mlp(0x1000, None, 0x1000, None)
    bad_dims = [sp.Dims(4100, 32000, 4, 512, 1e-5, 0.5),     # d not a multiple of 8
                sp.Dims(4096, 32000, 0, 512, 1e-5, 0.5),     # K < 1
                sp.Dims(4096, 32000, 17, 512, 1e-5, 0.5),    # K > KMAX
                sp.Dims(4096, 32000, 4, 4096, 1e-5, 0.5),    # H > HMAX
                sp.Dims(4096, 0, 4, 512, 1e-5, 0.5),         # V < 1
                sp.Dims(4096, 32000, 4, 512, -1.0, 0.5)]     # eps < 0
    other = C.c_void_p(0x2000)

    def predict(dm=None, B=1, hidden=fake, mlp_=C.byref(mlp), probs=other, prev=fake):
        return lib.specee_predict(dm, B, hidden, fake, fake, fake, prev, mlp_, None, fake, probs, fake, fake, None)

    ok = sp.Dims(4096, 32000, 4, 512, 1e-5, 0.5)
    for dm in bad_dims:
        assert predict(C.byref(dm)) == -1
    assert predict(None) == -1
    assert predict(C.byref(ok), B=-1) == -1
    assert predict(C.byref(ok), hidden=None) == -1
    assert predict(C.byref(ok), hidden=odd) == -2
    assert predict(C.byref(ok), mlp_=None) == -1
    assert predict(C.byref(ok), probs=fake, prev=fake) == -1          # probs aliases prev_probs
    assert lib.specee_predict(C.byref(ok), 0, None, None, None, None, None, None, None, None, None, None, None,
                              None) == 0
    # quantised rows: group must be a multiple of 8 that divides d; code words 4-byte aligned
    def q4(group=128, B=1, q=fake, probs=other):
        return lib.specee_predict_q4(C.byref(ok), B, fake, fake, q, fake, fake, group, fake, fake, C.byref(mlp), None,
                                     fake, probs, fake, fake, None)
    assert q4(group=12) == -1 and q4(group=4) == -1 and q4(group=4096 * 2) == -1 and q4(B=-1) == -1
    assert q4(q=None) == -1 and q4(probs=fake) == -1 and q4(q=C.c_void_p(fake.value + 2)) == -2
    assert q4(B=0, q=None) == 0
    # tree: limits and workspace
    args = (fake,) * 3 + (fake, None, fake, C.byref(mlp)) + (fake,) * 4 + (other,) + (fake,) * 2 + (None,)
    assert lib.specee_predict_tree(C.byref(ok), 1, 2000, 64, *args, fake, C.c_size_t(1 << 30), None) == -1  # N*K>4096
    assert lib.specee_predict_tree(C.byref(ok), 1, 60, 5000, *args, fake, C.c_size_t(1 << 30), None) == -1  # Mcap
    assert lib.specee_predict_tree(C.byref(ok), 1, 60, 64, *args, fake, C.c_size_t(16), None) == -3
    assert lib.specee_predict_tree(C.byref(ok), 1, 60, 64, *args, None, C.c_size_t(0), None) == -3
    args_path = (fake,) * 3 + (fake, None, fake, C.byref(mlp)) + (fake,) * 4 + (other,) + (fake,) * 2 + (fake,)
    assert lib.specee_predict_tree(C.byref(ok), 1, 60, 64, *args_path, fake, C.c_size_t(1 << 30), None) == -1
    # the entry point on static scratch: the same argument checks, made before anything touches a GPU
    assert lib.specee_predict_tree_static(C.byref(ok), 1, 2000, 64, *args, None) == -1
    assert lib.specee_predict_tree_static(C.byref(ok), 1, 60, 5000, *args, None) == -1
    assert lib.specee_predict_tree_static(C.byref(ok), 1, 60, 64, *args_path, None) == -1
    assert lib.specee_predict_tree_static(C.byref(ok), 0, 60, 64, *args, None) == 0
    assert lib.lm_head_gemv(C.byref(ok), 1, fake, fake, odd, fake, None, C.c_size_t(0), None) == -2
    assert lib.specee_verify(C.byref(ok), 1, fake, fake, fake, fake, None, None, fake, fake, fake, None,
                             C.c_size_t(0), None) == -3


def test_workspace_sizes(sp):
    dm = sp.Dims(4096, 32000, 4, 512, 1e-5, 0.5)
    assert sp.workspace_bytes(sp.OP_PREDICT, dm, 16) == 0
    assert sp.workspace_bytes(sp.OP_LM_HEAD, dm, 64) == 0
    one = sp.workspace_bytes(sp.OP_PREDICT_TREE, dm, 60, 64)
    # 16 d-slices of partial sums [60][64] fp32 plus the partial sums of squares, or (n could be 60 trees of
    # one node) 256 d-slice workgroups' accumulators of four row tiles, whichever is larger
    assert one >= 16 * 60 * 64 * 4 + 16 * 60 * 4 and one >= 256 * 256 * 4 * 16 and one < 5 << 20
    assert sp.workspace_bytes(sp.OP_PREDICT_TREE, dm, 16, 64) < 2 * 16 * 16 * 64 * 4     # too few nodes for that
    assert sp.workspace_bytes(sp.OP_PREDICT_TREE, dm, 6000, 64) > 4 * one
    assert sp.workspace_bytes(sp.OP_VERIFY, dm, 1) > 0
    with pytest.raises(sp.SpeceeError):
        sp.workspace_bytes(sp.OP_PREDICT_TREE, dm, 60, 0)
    with pytest.raises(sp.SpeceeError):
        sp.workspace_bytes(99, dm, 1)


def test_scheduler_matches_oracle(sp, oracle):
    rng = np.random.default_rng(11)
    L, Q, R, T = 32, 5, 2, 80
    seq = np.clip(np.round(rng.normal(22, 3, T)), 0, L - 1).astype(np.int32)
    off = np.zeros(L, np.int32); off[[20, 24, 28]] = 1
    ref_active, ref_counters = oracle.schedule(seq, L=L, Q=Q, radius=R, offline_mask=off)
    s = sp.Scheduler(L, Q, R, offline_mask=off)
    n_active = []
    for t in range(T):
        a = s.active()
        assert a == ref_active[t].tolist()
        assert s.counters() == ref_counters[t].tolist()
        n_active.append(sum(a))
        s.push(int(seq[t]))
    assert 3 <= np.mean(n_active) < L
    with pytest.raises(sp.SpeceeError):
        s.push(L)
    with pytest.raises(sp.SpeceeError):
        sp.Scheduler(1000)
