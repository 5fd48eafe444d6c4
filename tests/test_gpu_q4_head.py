"""GPU parity: the full-vocabulary head and the verification step on the 4-bit group-quantised LM head
(lm_head_gemv_q4, specee_verify_q4) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2504_08850_amd import synth

from parity import close, dev, host
from test_gpu_q4 import case, words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    specee.lib()
    return specee


def qdev(t):
    return words(t["q"]), dev(t["scales"]), dev(t["zeros"])


@pytest.mark.parametrize("d,V,N,group", [
    (64, 50, 3, 16),        # word-per-lane path (group not a multiple of 32)
    (1040, 301, 2, 104),    # ragged: 130 words per row, groups of 13 words
    (4096, 515, 1, 128),    # the 7B row: chunks of 32 elements, four rows per wavefront with a ragged tail
    (8192, 300, 2, 128),
    (2048, 1037, 5, 32),    # one chunk per group
    (8192, 77, 1, 64),      # 128 groups per row: more than one zero-point term per lane
    (16384, 40, 1, 128),    # largest hidden size (more than 64 KB of LDS for x)
    (8, 1, 1, 8),           # smallest everything
])
def test_lm_head_q4_shapes(sp, oracle, d, V, N, group):
    t = case(d + V, d, V, 1, 8, N, group, False)
    ref = oracle.lm_head_gemv_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], group)
    got = host(sp.lm_head_gemv_q4(dev(t["hidden"]), dev(t["gamma"]), *qdev(t), group))
    close(got, ref, 1.0, f"lm_head_q4 d={d} V={V} group={group}")


def test_lm_head_q4_unaligned_codes_take_the_word_path(sp, oracle):
    t = case(5, 4096, 130, 1, 8, 2, 128, False)
    ref = oracle.lm_head_gemv_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], 128)
    buf = torch.zeros(t["q"].size + 1, dtype=torch.int32, device="cuda")
    buf[1:] = words(t["q"]).flatten()
    qd = buf[1:].view(t["q"].shape)                  # 4 bytes past a 16-byte boundary
    assert qd.data_ptr() % 16 == 4
    got = host(sp.lm_head_gemv_q4(dev(t["hidden"]), dev(t["gamma"]), qd, dev(t["scales"]), dev(t["zeros"]), 128))
    close(got, ref, 1.0, "lm_head_q4 unaligned codes")


def run_verify(sp, t, ids, **kw):
    out = sp.verify_q4(dev(t["hidden"]), dev(t["gamma"]), *qdev(t), t["group"], dev(ids), **kw)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in out.items()}


def check_verify(got, full, ids, what, live=None):
    """full: the oracle's logits [N][V].  The arg-max must be the oracle's wherever the runner-up is further away
    than the tolerance; otherwise any of the near-tied tokens is accepted."""
    N = full.shape[0]
    for n in range(N):
        if live is not None and not live[n]:
            assert got["token"][n] == -1 and got["hit"][n] == 0 and got["max_logit"][n] == 0, what
            continue
        order = np.argsort(-full[n], kind="stable")
        top = full[n, order[0]]
        tol = 2e-3 * max(1.0, abs(top))
        near = set(int(v) for v in order[:8] if top - full[n, v] <= tol)
        if len(near) == 1:
            assert got["token"][n] == order[0], (what, n)
        else:
            assert int(got["token"][n]) in near, (what, n)
        assert abs(got["max_logit"][n] - top) <= tol, what
        assert got["hit"][n] == int(got["token"][n] in ids[n]), what


@pytest.mark.parametrize("d,V,N,K,group", [(64, 37, 1, 3, 16), (1040, 1001, 2, 4, 104), (4096, 515, 5, 4, 128),
                                           (2048, 4100, 9, 8, 32), (8, 1, 1, 1, 8)])
def test_verify_q4_small(sp, oracle, d, V, N, K, group):
    t = case(d + V + N, d, V, min(K, V), 8, N, group, False)
    full = oracle.lm_head_gemv_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], group)
    ids = t["ids"].copy()
    ids[::2, 0] = full.argmax(axis=1)[::2]          # half of the states hit
    got = run_verify(sp, t, ids)
    check_verify(got, full, ids, f"verify_q4 d={d} V={V} N={N}")
    ref = oracle.verify_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], group, ids)
    assert np.array_equal(ref["token"], full.argmax(axis=1))
    assert got["hit"].sum() > 0 or N == 1


def test_verify_q4_tie_goes_to_lowest_id(sp):
    t = case(3, 256, 40, 2, 8, 1, 64, False)
    q, s, z = t["q"].copy(), t["scales"].copy(), t["zeros"].copy()
    # three identical rows that win by construction: codes follow the sign of x, largest scale
    x = t["hidden"][0].astype(np.float64) * t["gamma"].astype(np.float64)
    codes = np.where(x > 0, 15, 0).astype(np.uint32)
    wrow = (codes.reshape(-1, 8) << (4 * np.arange(8, dtype=np.uint32))).sum(axis=1, dtype=np.uint32)
    for v in (31, 7, 19):
        q[v], s[v], z[v] = wrow, np.float16(1.0), np.float16(7.0)
    t2 = dict(t, q=q, scales=s, zeros=z)
    got = run_verify(sp, t2, np.array([[19, 5]], np.int32))
    assert got["token"][0] == 7 and got["hit"][0] == 0
    got = run_verify(sp, t2, np.array([[19, 7]], np.int32))
    assert got["token"][0] == 7 and got["hit"][0] == 1


def test_verify_q4_gate_and_done_flags(sp, oracle):
    N = 6
    t = case(11, 1040, 301, 4, 8, N, 104, False)
    full = oracle.lm_head_gemv_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], t["group"])
    ids = t["ids"].copy()
    ids[:, 1] = full.argmax(axis=1)                  # every verified state hits
    gate = np.array([1, 0, 1, 1, 0, 1], np.int32)
    done = np.array([0, 0, 1, 0, 0, 0], np.int32)
    done_d = dev(done)
    got = run_verify(sp, t, ids, gate=dev(gate), done=done_d)
    live = (gate != 0) & (done == 0)
    check_verify(got, full, ids, "verify_q4 gated", live=live)
    assert np.array_equal(host(done_d), np.where(live, 1, done))     # hits are recorded, the rest untouched
    none = run_verify(sp, t, ids, gate=dev(np.zeros(N, np.int32)))   # nothing gated in: no pass over the head
    assert np.all(none["token"] == -1) and not none["hit"].any()


def test_q4_head_llama7b_shape_and_the_predictor_reads_its_rows(sp, oracle):
    """32000 x 4096 head quantised in groups of 128: every logit against the oracle, the verification on top, and
    the quantised-rows predictor's logits are this head's logits at the ids."""
    c = synth.CONFIGS["C1"]
    lm_h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
    q, s, z = synth.quantize_q4(lm_h, 128)
    t1 = synth.make("C1", seed=2, lm=lm_h)
    qd = (words(q), dev(s), dev(z))
    oracle.set_threads(8)
    full = oracle.lm_head_gemv_q4(t1["hidden"], t1["gamma"], q, s, z, 128)
    oracle.set_threads(1)
    got = host(sp.lm_head_gemv_q4(dev(t1["hidden"]), dev(t1["gamma"]), *qd, 128))
    w = close(got, full, 1.0, "lm_head_q4 32000x4096")
    print("lm_head_q4 32000x4096 worst", w)
    ids = t1["ids"].copy()
    ids[0, 2] = int(full[0].argmax())
    v = sp.verify_q4(dev(t1["hidden"]), dev(t1["gamma"]), *qd, 128, dev(ids))
    torch.cuda.synchronize()
    check_verify({k: host(x) for k, x in v.items()}, full, ids, "verify_q4 32000x4096")
    assert host(v["hit"])[0] == 1
    p = sp.predict_q4(dev(t1["hidden"]), dev(t1["gamma"]), *qd, 128, dev(ids), dev(t1["prev_probs"]), dev(t1["W1"]),
                      dev(t1["w2"]))
    torch.cuda.synchronize()
    close(host(p["logits"]), np.take_along_axis(got, ids, axis=1), 1.0, "quantised predictor vs quantised head")


def test_q4_head_argument_errors(sp):
    t = case(1, 64, 20, 2, 8, 1, 16, False)
    a = (dev(t["hidden"]), dev(t["gamma"]), *qdev(t))
    five = torch.ones((20, 5), dtype=torch.float16, device="cuda")
    with pytest.raises(sp.SpeceeError) as ei:
        sp.lm_head_gemv_q4(a[0], a[1], a[2], five, five, 12)
    assert ei.value.code == -1                       # group must be a multiple of 8 that divides d
    with pytest.raises(sp.SpeceeError) as ei:
        sp.verify_q4(*a, 16, dev(t["ids"]), workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == -3
