"""GPU parity: specee_predict_q4 (the predictor on a 4-bit group-quantised LM head) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2504_08850_amd import synth

from parity import check_scored, close, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    specee.lib()
    return specee


def words(q):
    """uint32 words -> the int32 tensor the binding takes (same bits)."""
    return dev(np.ascontiguousarray(q).view(np.int32))


def case(seed, d, V, K, H, B, group, bias):
    rng = np.random.default_rng(seed)
    w = (0.05 * rng.standard_normal((V, d))).astype(np.float16)
    q, scales, zeros = synth.quantize_q4(w, group)
    return dict(
        hidden=rng.standard_normal((B, d)).astype(np.float16),
        gamma=(1 + 0.05 * rng.standard_normal(d)).astype(np.float16),
        q=q, scales=scales, zeros=zeros, group=group,
        ids=np.stack([rng.choice(V, K, replace=False) for _ in range(B)]).astype(np.int32),
        prev_probs=rng.dirichlet(np.ones(K), size=B).astype(np.float32),
        W1=(0.3 * rng.standard_normal((H, 3 * K))).astype(np.float16),
        w2=(0.3 * rng.standard_normal(H)).astype(np.float16),
        b1=(0.2 * rng.standard_normal(H)).astype(np.float16) if bias else None,
        b2=(0.2 * rng.standard_normal(1)).astype(np.float16) if bias else None)


def run(sp, t, qd=None, **kw):
    qd = qd or (words(t["q"]), dev(t["scales"]), dev(t["zeros"]))
    out = sp.predict_q4(dev(t["hidden"]), dev(t["gamma"]), *qd, t["group"], dev(t["ids"]), dev(t["prev_probs"]),
                        dev(t["W1"]), dev(t["w2"]), dev(t["b1"]), dev(t["b2"]), **kw)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in out.items()}


def ref(oracle, t, **kw):
    return oracle.predict_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], t["group"], t["ids"],
                             t["prev_probs"], t["W1"], t["w2"], t["b1"], t["b2"], **kw)


@pytest.mark.parametrize("d,V,K,H,B,group,bias", [
    (64, 50, 3, 40, 5, 16, True),        # tiny, K odd
    (1040, 301, 4, 512, 7, 104, False),  # ragged: 130 vectors, group of 13 words
    (4096, 515, 4, 512, 9, 128, True),   # the 7B shape: one word per thread and row
    (8192, 300, 8, 512, 3, 128, False),  # two vectors per thread
    (12288, 99, 2, 64, 2, 64, True),     # more vectors than the unrolled part holds
    (256, 77, 16, 2048, 4, 8, True),     # K = KMAX, H = HMAX, smallest group
    (8, 3, 1, 1, 1, 8, False),           # smallest everything
])
def test_q4_shapes(sp, oracle, d, V, K, H, B, group, bias):
    t = case(d + K, d, V, K, H, B, group, bias)
    check_scored(run(sp, t), ref(oracle, t), 0.5, f"q4 d={d} K={K} group={group}")


def test_q4_llama7b_shape_done_flags_and_invalid_ids(sp, oracle):
    c = synth.CONFIGS["C1"]
    lm_h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
    q, scales, zeros = synth.quantize_q4(lm_h, 128)
    qd = (words(q), dev(scales), dev(zeros))
    B = 48
    base = synth.make("C1", seed=5, lm=lm_h)
    t = dict(base, hidden=synth.hidden(B, c.d, 31), ids=synth.ids_uniform_distinct(B, c.K, c.V, 32),
             prev_probs=synth.prob_rows(B, c.K, 33), q=q, scales=scales, zeros=zeros, group=128)
    r = ref(oracle, t)
    got = run(sp, t, qd)
    e = check_scored(got, r, c.threshold, "q4 C1 shape")
    print("q4 C1 worst relative errors", e)
    # the quantised logits stay near the fp16 ones: errors of up to half a step (~0.004) per element with
    # random signs add up to a standard deviation of about 0.15 over 4096 elements
    full = oracle.predict(t["hidden"], t["gamma"], lm_h, t["ids"], t["prev_probs"], t["W1"], t["w2"])
    dq = np.abs(r["logits"] - full["logits"])
    assert 0.02 < dq.std() < 0.4 and dq.max() < 1.0
    # done tokens are skipped, the rest unchanged
    done = (np.arange(B) % 3 == 0).astype(np.int32)
    got_d = run(sp, t, qd, done=dev(done))
    on = done == 0
    for k in ("logits", "probs", "scores", "exit"):
        assert np.array_equal(got_d[k][on], got[k][on]), k
    assert np.all(got_d["logits"][~on] == 0) and np.all(got_d["scores"][~on] == 0) and np.all(got_d["exit"][~on] == 0)
    assert np.array_equal(got_d["probs"][~on], t["prev_probs"][~on])
    # an id outside the vocabulary poisons its token only
    bad = dict(t, ids=t["ids"].copy())
    bad["ids"][7, 2] = c.V
    bad["ids"][9, 0] = -1
    got_b = run(sp, bad, qd)
    assert np.isnan(got_b["scores"][7]) and np.isnan(got_b["scores"][9]) and got_b["exit"][7] == 0
    keep = np.ones(B, bool); keep[[7, 9]] = False
    assert np.array_equal(got_b["scores"][keep], got["scores"][keep])


def test_q4_batch_of_8000_sampled_tokens(sp, oracle):
    c = synth.CONFIGS["C1"]
    lm_h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
    q, scales, zeros = synth.quantize_q4(lm_h, 128)
    B = 8000
    rng = np.random.default_rng(8)
    base = synth.make("C1", lm=lm_h)
    t = dict(base, hidden=rng.standard_normal((B, c.d), dtype=np.float32).astype(np.float16),
             ids=rng.permutation(c.V)[:B * c.K].reshape(B, c.K).astype(np.int32),
             prev_probs=synth.prob_rows(B, c.K, 9), q=q, scales=scales, zeros=zeros, group=128)
    got = run(sp, t)
    pick = np.unique(np.concatenate([[0, B - 1], rng.integers(0, B, 64)]))
    sub = dict(t, hidden=t["hidden"][pick], ids=t["ids"][pick], prev_probs=t["prev_probs"][pick])
    check_scored({k: v[pick] for k, v in got.items()}, ref(oracle, sub), c.threshold, "q4 B=8000 sampled")
    assert np.all(np.isfinite(got["scores"])) and np.allclose(got["probs"].sum(axis=1), 1, atol=1e-5)


@pytest.mark.parametrize("d,V,group", [
    (8192, 600, 128),   # 32-element chunks, 256 threads
    (4096, 500, 32),    # 32-element chunks, 128 threads, smallest group that allows them
    (2080, 400, 32),    # 65 chunks: half of the threads hold a clamped, silenced duplicate
    (8192, 300, 64),
    (4096, 500, 8),     # group too small for chunks: one word per thread and row
    (1040, 300, 104),   # group not a multiple of 32
])
def test_q4_large_batch_formats(sp, oracle, d, V, group):
    """More than a thousand tokens per launch take the throughput shapes, whichever the format allows."""
    t = case(d + group, d, V, 4, 512, 1100, group, True)
    got = run(sp, t)
    pick = np.array([0, 1, 511, 1023, 1024, 1099])
    sub = dict(t, hidden=t["hidden"][pick], ids=t["ids"][pick], prev_probs=t["prev_probs"][pick])
    check_scored({k: v[pick] for k, v in got.items()}, ref(oracle, sub), 0.5, f"q4 d={d} group={group} B=1100")
    assert np.all(np.isfinite(got["scores"]))


def test_q4_large_batch_done_invalid_ids_and_unaligned_codes(sp, oracle):
    t = case(5, 4096, 300, 4, 512, 1100, 128, True)
    qd = (words(t["q"]), dev(t["scales"]), dev(t["zeros"]))
    got = run(sp, t, qd)
    # the same codes at an address that is only 4-byte aligned: the word-per-thread shape takes over
    flat = torch.empty(t["q"].size + 1, dtype=torch.int32, device="cuda")
    flat[1:] = qd[0].reshape(-1)
    shifted = flat[1:].reshape(qd[0].shape)
    assert shifted.data_ptr() % 16 == 4
    got_s = run(sp, t, (shifted, qd[1], qd[2]))
    pick = np.array([0, 3, 600, 1099])
    sub = dict(t, hidden=t["hidden"][pick], ids=t["ids"][pick], prev_probs=t["prev_probs"][pick])
    r = ref(oracle, sub)
    check_scored({k: v[pick] for k, v in got.items()}, r, 0.5, "q4 B=1100 aligned")
    check_scored({k: v[pick] for k, v in got_s.items()}, r, 0.5, "q4 B=1100 codes at a 4-byte-aligned address")
    assert np.allclose(got_s["logits"], got["logits"], rtol=1e-4, atol=1e-4)  # same values up to summation order
    # done tokens are skipped, the rest unchanged
    done = (np.arange(1100) % 5 == 0).astype(np.int32)
    got_d = run(sp, t, qd, done=dev(done))
    on = done == 0
    for k in ("logits", "probs", "scores", "exit"):
        assert np.array_equal(got_d[k][on], got[k][on]), k
    assert np.all(got_d["logits"][~on] == 0) and np.all(got_d["scores"][~on] == 0) and np.all(got_d["exit"][~on] == 0)
    assert np.array_equal(got_d["probs"][~on], t["prev_probs"][~on])
    # an id outside the vocabulary poisons its token only
    bad = dict(t, ids=t["ids"].copy())
    bad["ids"][7, 2] = 300
    bad["ids"][1024, 0] = -1
    got_b = run(sp, bad, qd)
    assert np.isnan(got_b["scores"][7]) and np.isnan(got_b["scores"][1024]) and got_b["exit"][7] == 0
    keep = np.ones(1100, bool); keep[[7, 1024]] = False
    assert np.array_equal(got_b["scores"][keep], got["scores"][keep])


def test_q4_argument_errors(sp):
    t = case(1, 64, 20, 2, 8, 2, 16, False)
    qd = (words(t["q"]), dev(t["scales"]), dev(t["zeros"]))
    for group in (12, 4, 48):            # not a multiple of 8 / too small / does not divide d
        with pytest.raises(sp.SpeceeError):
            sp.predict_q4(dev(t["hidden"]), dev(t["gamma"]), qd[0], dev(np.ones((20, 64 // group), np.float16)),
                          dev(np.ones((20, 64 // group), np.float16)), group, dev(t["ids"]), dev(t["prev_probs"]),
                          dev(t["W1"]), dev(t["w2"]))
