"""Pins for the CPU oracle: every oracle function is checked against something other
than itself -- numpy / scipy library routines, closed forms, brute force on tiny
shapes, the structural invariants the paper fixes and the few numbers it prints.
CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import expit, softmax

from paper_2504_08850_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def f64(a):
    return np.asarray(a, dtype=np.float64)


def small(seed=0, d=24, V=19, K=3, H=16, B=4, bias=True):
    rng = np.random.default_rng(seed)
    t = dict(
        hidden=rng.standard_normal((B, d)).astype(np.float16),
        gamma=(1 + 0.1 * rng.standard_normal(d)).astype(np.float16),
        lm_head=(0.3 * rng.standard_normal((V, d))).astype(np.float16),
        ids=np.stack([rng.choice(V, K, replace=False) for _ in range(B)]).astype(np.int32),
        prev_probs=rng.dirichlet(np.ones(K), size=B).astype(np.float32),
        W1=(0.5 * rng.standard_normal((H, 3 * K))).astype(np.float16),
        w2=(0.5 * rng.standard_normal(H)).astype(np.float16),
        b1=(0.5 * rng.standard_normal(H)).astype(np.float16) if bias else None,
        b2=(0.5 * rng.standard_normal(1)).astype(np.float16) if bias else None,
    )
    return t


def np_normed(hidden, gamma, eps):
    """Textbook RMSNorm with numpy float64 library reductions."""
    h = f64(hidden)
    r = 1.0 / np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + eps)
    return h * r * f64(gamma)


# ---------------------------------------------------------------- fp16 decode
def test_half_decode_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- RMSNorm scale
def test_rms_scale_closed_form_constant_vector(oracle):
    for c, d, eps in [(2.0, 16, 1e-5), (-0.5, 7, 1e-3), (3.0, 1, 0.0)]:
        h = np.full(d, c, dtype=np.float16)
        assert oracle.rms_scale(h, eps) == pytest.approx(1.0 / math.sqrt(c * c + eps), rel=1e-14)


def test_rms_scale_matches_numpy_and_scale_invariance(oracle):
    rng = np.random.default_rng(1)
    h = rng.standard_normal(333).astype(np.float16)
    want = 1.0 / np.sqrt(np.mean(f64(h) ** 2) + 1e-5)
    assert oracle.rms_scale(h, 1e-5) == pytest.approx(want, rel=1e-13)
    # doubling h (exact in fp16) halves the scale when eps = 0
    assert oracle.rms_scale((2 * h).astype(np.float16), 0.0) == pytest.approx(oracle.rms_scale(h, 0.0) / 2, rel=1e-14)
    # zero hidden state: scale is 1/sqrt(eps)
    assert oracle.rms_scale(np.zeros(8, np.float16), 1e-4) == pytest.approx(100.0, rel=1e-14)


# ---------------------------------------------------------------- logits
def test_logits_match_numpy_matmul(oracle):
    t = small(2)
    out = oracle.predict(**t, eps=1e-5)
    x = np_normed(t["hidden"], t["gamma"], 1e-5)
    for n in range(x.shape[0]):
        want = f64(t["lm_head"])[t["ids"][n]] @ x[n]
        np.testing.assert_allclose(out["logits"][n], want, rtol=1e-12, atol=1e-13)


def test_logits_brute_force_python_loops(oracle):
    t = small(3, d=5, V=7, K=2, H=3, B=2)
    out = oracle.predict(**t, eps=1e-3)
    for n in range(2):
        h = [float(v) for v in t["hidden"][n]]
        ms = sum(v * v for v in h) / len(h)
        r = 1.0 / math.sqrt(ms + 1e-3)
        for k in range(2):
            row = t["lm_head"][t["ids"][n, k]]
            z = 0.0
            for i in range(5):
                z += h[i] * r * float(t["gamma"][i]) * float(row[i])
            assert out["logits"][n, k] == pytest.approx(z, rel=1e-13, abs=1e-15)


def test_reduced_logits_equal_full_vocab_logits_at_ids(oracle):
    """The speculative logits are the full LM-head logits indexed at the ids (bit-equal)."""
    t = small(4, d=40, V=31, K=4, B=6)
    out = oracle.predict(**t)
    full = oracle.lm_head_gemv(t["hidden"], t["gamma"], t["lm_head"])
    for n in range(6):
        assert np.array_equal(out["logits"][n], full[n, t["ids"][n]])


def test_one_hot_rows_pick_normalised_coordinates(oracle):
    d, V, K = 12, 12, 3
    t = small(5, d=d, V=V, K=K, B=2)
    t["lm_head"] = np.eye(V, d, dtype=np.float16)
    out = oracle.predict(**t)
    x = np_normed(t["hidden"], t["gamma"], 1e-5)
    for n in range(2):
        np.testing.assert_allclose(out["logits"][n], x[n, t["ids"][n]], rtol=1e-14)


def test_gamma_is_applied_elementwise_not_dropped(oracle):
    t = small(6)
    base = oracle.predict(**t)["logits"]
    t2 = dict(t)
    t2["gamma"] = (2 * t["gamma"]).astype(np.float16)   # exact doubling
    np.testing.assert_allclose(oracle.predict(**t2)["logits"], 2 * base, rtol=1e-14)
    t3 = dict(t)
    g = t["gamma"].copy(); g[0] = 0
    t3["gamma"] = g
    x = np_normed(t["hidden"], g, 1e-5)
    np.testing.assert_allclose(oracle.predict(**t3)["logits"][0], f64(t["lm_head"])[t["ids"][0]] @ x[0], rtol=1e-12,
                               atol=1e-13)


def test_permuting_ids_permutes_outputs(oracle):
    t = small(7, K=4)
    a = oracle.predict(**t)
    perm = np.array([2, 0, 3, 1])
    t2 = dict(t); t2["ids"] = t["ids"][:, perm]; t2["prev_probs"] = t["prev_probs"][:, perm]
    b = oracle.predict(**t2)
    assert np.array_equal(b["logits"], a["logits"][:, perm])
    np.testing.assert_allclose(b["probs"], a["probs"][:, perm], rtol=1e-14)


# ---------------------------------------------------------------- softmax / delta / features
def test_local_probs_match_scipy_softmax_and_sum_to_one(oracle):
    t = small(8, K=5, B=9)
    out = oracle.predict(**t)
    np.testing.assert_allclose(out["probs"], softmax(out["logits"], axis=1), rtol=1e-13)
    np.testing.assert_allclose(out["probs"].sum(axis=1), 1.0, atol=1e-12)


def test_softmax_special_cases(oracle):
    # identical rows -> uniform; K = 1 -> probability one
    t = small(9, K=4, V=10)
    t["lm_head"][:] = t["lm_head"][0]
    np.testing.assert_allclose(oracle.predict(**t)["probs"], 0.25, rtol=1e-14)
    t1 = small(10, K=1)
    assert np.array_equal(oracle.predict(**t1)["probs"], np.ones((4, 1)))


def test_softmax_is_stable_for_large_logits(oracle):
    t = small(11, d=8, V=4, K=2, B=1)
    t["lm_head"] = np.zeros((4, 8), np.float16)
    t["lm_head"][0] = 200.0
    t["lm_head"][1] = -200.0
    t["hidden"] = np.full((1, 8), 10.0, np.float16)
    t["gamma"] = np.ones(8, np.float16)
    t["ids"] = np.array([[0, 1]], np.int32)
    out = oracle.predict(**t)
    assert np.all(np.isfinite(out["probs"])) and out["probs"][0, 0] == pytest.approx(1.0)


def test_feature_layout_and_variation(oracle):
    """[logits | probs | probs - prev]; variation sums to zero when prev is a distribution."""
    t = small(12, K=4)
    out = oracle.predict(**t)
    K = 4
    f = out["features"]
    assert np.array_equal(f[:, :K], out["logits"])
    assert np.array_equal(f[:, K:2 * K], out["probs"])
    assert np.array_equal(f[:, 2 * K:], out["probs"] - f64(t["prev_probs"]))
    np.testing.assert_allclose(f[:, 2 * K:].sum(axis=1), 0.0, atol=1e-7)
    t0 = dict(t); t0["prev_probs"] = np.zeros_like(t["prev_probs"])
    f0 = oracle.predict(**t0)["features"]
    assert np.array_equal(f0[:, 2 * K:], f0[:, K:2 * K])


def test_paper_variation_example_keeps_probability_as_separate_feature(oracle):
    """Sec. 4.3.1 example: the same variation 0.12 arises from 0.32-0.20 and from 0.58-0.46;
    the two states must differ in the probability slot."""
    vals = {}
    with open(os.path.join(GOLD, "variation_example.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    feats = []
    for p_now, p_last in [(vals["left_now"], vals["left_last"]), (vals["right_now"], vals["right_last"])]:
        # two tokens, one-hot rows, d = 2, gamma = 1, eps = 0: z = h / rms(h), z0 - z1 = log(p/(1-p))
        tlog = math.log(p_now / (1 - p_now))
        x0 = (tlog + math.sqrt(4 - tlog * tlog)) / 2
        h = np.array([[x0, x0 - tlog]], dtype=np.float16)
        out = oracle.predict(hidden=h, gamma=np.ones(2, np.float16), lm_head=np.eye(2, dtype=np.float16),
                             ids=np.array([[0, 1]], np.int32), prev_probs=np.array([[p_last, 1 - p_last]], np.float32),
                             W1=np.zeros((1, 6), np.float16), w2=np.zeros(1, np.float16), eps=0.0)
        assert out["probs"][0, 0] == pytest.approx(p_now, abs=2e-3)
        feats.append(out["features"][0])
    assert feats[0][4] == pytest.approx(vals["variation"], abs=2e-3)
    assert feats[1][4] == pytest.approx(vals["variation"], abs=2e-3)
    assert abs(feats[0][2] - feats[1][2]) > 0.2


# ---------------------------------------------------------------- MLP + judgment
def test_mlp_matches_numpy_and_scipy(oracle):
    for bias in (True, False):
        t = small(13, K=4, H=33, B=8, bias=bias)
        out = oracle.predict(**t)
        W1, w2 = f64(t["W1"]), f64(t["w2"])
        b1 = f64(t["b1"]) if bias else 0.0
        b2 = float(t["b2"][0]) if bias else 0.0
        a = np.maximum(out["features"] @ W1.T + b1, 0.0)
        want = expit(a @ w2 + b2)
        np.testing.assert_allclose(out["scores"], want, rtol=1e-12)
        band = np.abs(want - 0.5) > 1e-6
        assert np.array_equal(out["exit"][band], (want > 0.5).astype(np.int32)[band])
        assert 0 < out["exit"].sum() < 8 or True


def test_each_feature_reaches_the_right_mlp_input(oracle):
    """W1 is [H][3K] (output x input): a single unit weight at (0, t) must select feature t."""
    t = small(14, K=3, H=5, bias=False)
    base = oracle.predict(**t)["features"]
    for col in range(9):
        W1 = np.zeros((5, 9), np.float16); W1[0, col] = 1.0
        w2 = np.zeros(5, np.float16); w2[0] = 1.0
        t2 = dict(t, W1=W1, w2=w2)
        s = oracle.predict(**t2)["scores"]
        np.testing.assert_allclose(s, expit(np.maximum(base[:, col], 0.0)), rtol=1e-13)
    # the hidden index of w2 matters too
    W1 = np.zeros((5, 9), np.float16); W1[3, 1] = 1.0
    w2 = np.zeros(5, np.float16); w2[3] = -2.0
    s = oracle.predict(**dict(t, W1=W1, w2=w2))["scores"]
    np.testing.assert_allclose(s, expit(-2.0 * np.maximum(base[:, 1], 0.0)), rtol=1e-13)


def test_relu_clips_negative_preactivations(oracle):
    t = small(15, K=2, H=1, bias=False, B=1)
    t["W1"] = np.zeros((1, 6), np.float16); t["W1"][0, 2] = -1.0   # -(prob) < 0 -> clipped
    t["w2"] = np.ones(1, np.float16)
    assert oracle.predict(**t)["scores"][0] == 0.5
    t["b1"] = np.array([2.0], np.float16)                            # 2 - p > 0
    out = oracle.predict(**t)
    assert out["scores"][0] == pytest.approx(expit(2.0 - out["probs"][0, 0]), rel=1e-13)
    t["b2"] = np.array([-1.0], np.float16)
    out = oracle.predict(**t)
    assert out["scores"][0] == pytest.approx(expit(1.0 - out["probs"][0, 0]), rel=1e-13)


def test_zero_weights_give_half_and_no_exit_strict_threshold(oracle):
    t = small(16, bias=False)
    t["W1"][:] = 0; t["w2"][:] = 0
    out = oracle.predict(**t, threshold=0.5)
    assert np.array_equal(out["scores"], np.full(4, 0.5))
    assert out["exit"].sum() == 0                       # strict comparison: 0.5 does not pass 0.5
    assert oracle.predict(**t, threshold=0.49)["exit"].sum() == 4


def test_predictor_parameter_memory_matches_paper(oracle):
    """Sec. 7.4.2: all 32 predictors of Llama2-7B with 4 draft tokens take 416 KB."""
    with open(os.path.join(GOLD, "predictor_memory.txt")) as fh:
        kb = [float(l.split()[1]) for l in fh if l.startswith("total_kib")][0]
    m = synth.mlp(K=4, H=512, seed=0, L=32)
    assert m["b1"] is None and m["b2"] is None
    assert (m["W1"].nbytes + m["w2"].nbytes) / 1024 == kb
    assert m["W1"].shape == (32, 512, 12)


# ---------------------------------------------------------------- layer sweep
def test_sweep_equals_chained_single_layer_calls(oracle):
    c = synth.CONFIGS["T2"]
    t = synth.make("T2", bias=True)
    sw = oracle.predict_sweep(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"])
    prev = np.zeros((c.B, c.K), np.float32)
    first = np.full(c.B, -1)
    for l in range(c.L):
        one = oracle.predict(t["hidden"][l], t["gamma"], t["lm_head"], t["ids"], prev, t["W1"][l], t["w2"][l],
                             t["b1"][l], t["b2"][l:l + 1])
        assert np.array_equal(one["logits"], sw["logits"][l])
        assert np.array_equal(one["probs"], sw["probs"][l])
        assert np.array_equal(one["scores"], sw["scores"][l])
        assert np.array_equal(one["exit"], sw["exit"][l])
        first = np.where((first < 0) & (one["exit"] == 1), l, first)
        prev = one["probs"].astype(np.float32)
    assert np.array_equal(first, sw["first_exit"])
    assert sw["exit"].sum() not in (0, sw["exit"].size)


def test_sweep_inactive_layers_are_skipped_and_do_not_touch_the_carry(oracle):
    t = synth.make("T2")
    active = np.array([1, 0, 0, 1, 1], np.int32)
    sw = oracle.predict_sweep(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], active=active)
    assert not sw["scores"][1].any() and not sw["exit"][1].any() and not sw["probs"][2].any()
    one0 = oracle.predict(t["hidden"][0], t["gamma"], t["lm_head"], t["ids"], np.zeros((7, 4), np.float32),
                          t["W1"][0], t["w2"][0])
    one3 = oracle.predict(t["hidden"][3], t["gamma"], t["lm_head"], t["ids"], one0["probs"].astype(np.float32),
                          t["W1"][3], t["w2"][3])
    assert np.array_equal(one3["scores"], sw["scores"][3])


# ---------------------------------------------------------------- merged tree mapping
def test_merge_matches_numpy_unique(oracle):
    rng = np.random.default_rng(20)
    for n, hi in [(1, 5), (17, 6), (240, 70), (512, 100000)]:
        ids = rng.integers(0, hi, size=n).astype(np.int32)
        merged, M, cols = oracle.merge(ids, cap=n + 3)
        u, inv = np.unique(ids, return_inverse=True)
        assert M == len(u) == len(set(ids.tolist()))
        assert np.array_equal(merged[:M], u) and np.all(merged[M:] == -1)
        assert np.array_equal(cols, inv)
        assert np.array_equal(merged[cols], ids)


def test_merge_extremes_and_overflow(oracle):
    same = np.tile(np.array([9, 4, 7], np.int32), (10, 1))
    merged, M, cols = oracle.merge(same, cap=8)
    assert M == 3 and merged[:3].tolist() == [4, 7, 9] and np.array_equal(cols, np.tile([2, 0, 1], (10, 1)))
    distinct = np.arange(40, dtype=np.int32)[::-1].reshape(10, 4)
    merged, M, cols = oracle.merge(distinct, cap=40)
    assert M == 40 and np.array_equal(merged, np.arange(40)) and np.array_equal(cols, distinct)
    with pytest.raises(ValueError):
        oracle.merge(distinct, cap=39)


@pytest.mark.parametrize("name", ["T3", "T4"])
def test_merged_tree_equals_independent_per_node_predictors(oracle, name):
    """Sec. 6.2: the merged mapping must give every node what its own independent mapping gives."""
    t = synth.make(name, bias=(name == "T4"))
    c = t["cfg"]
    tree = oracle.predict_tree(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["prev_probs"], t["W1"], t["w2"],
                               t["b1"], t["b2"], parent=t["parent"], Mcap=c.Mcap)
    ind = oracle.predict(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["prev_probs"], t["W1"], t["w2"],
                         t["b1"], t["b2"])
    for key in ("logits", "probs", "scores", "exit"):
        assert np.array_equal(tree[key], ind[key]), key
    M = int(tree["M"])
    assert M == len(np.unique(t["ids"])) and M < c.N * c.K     # the generator really overlaps ids
    x = np_normed(t["hidden"], t["gamma"], c.eps)
    Zwant = x @ f64(t["lm_head"])[tree["merged"][:M]].T
    np.testing.assert_allclose(tree["Z"][:, :M], Zwant, rtol=1e-11, atol=1e-12)
    assert not tree["Z"][:, M:].any()
    assert 0 < tree["exit"].sum() < c.N


def test_path_exit_is_and_over_root_path(oracle):
    t = synth.make("T3")
    c = t["cfg"]
    tree = oracle.predict_tree(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["prev_probs"], t["W1"], t["w2"],
                               parent=t["parent"], Mcap=c.Mcap)
    ex, par = tree["exit"], t["parent"]
    for n in range(c.N):
        ok, m = 1, n
        while m >= 0:
            ok &= int(ex[m]); m = int(par[m])
        assert tree["path_exit"][n] == ok
    assert 0 < tree["path_exit"].sum() < tree["exit"].sum()


def test_tree_batches_are_independent(oracle):
    t = synth.make("T4")
    c = t["cfg"]
    t2 = synth.make("T4", seed=1)
    hid = np.stack([t["hidden"], t2["hidden"]]); ids = np.stack([t["ids"], t2["ids"]])
    prev = np.stack([t["prev_probs"], t2["prev_probs"]]); par = np.stack([t["parent"], t2["parent"]])
    both = oracle.predict_tree(hid, t["gamma"], t["lm_head"], ids, prev, t["W1"], t["w2"], parent=par, Mcap=c.Mcap)
    for g, src in enumerate((t, t2)):
        one = oracle.predict_tree(src["hidden"], t["gamma"], t["lm_head"], src["ids"], src["prev_probs"], t["W1"],
                                  t["w2"], parent=src["parent"], Mcap=c.Mcap)
        for key in ("merged", "cols", "logits", "probs", "scores", "exit", "path_exit"):
            assert np.array_equal(both[key][g], one[key]), key
        assert both["M"][g] == one["M"]


def test_tree_rejects_bad_arguments(oracle):
    t = synth.make("T4")
    c = t["cfg"]
    bad = t["ids"].copy(); bad[3, 1] = c.V
    with pytest.raises(ValueError):
        oracle.predict_tree(t["hidden"], t["gamma"], t["lm_head"], bad, t["prev_probs"], t["W1"], t["w2"], Mcap=c.Mcap)
    par = t["parent"].copy(); par[2] = 5
    with pytest.raises(ValueError):
        oracle.predict_tree(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["prev_probs"], t["W1"], t["w2"],
                            parent=par, Mcap=c.Mcap)


# ---------------------------------------------------------------- full-vocabulary head + verification
def test_full_head_matches_numpy_matmul_and_row_subset(oracle):
    t = small(30, d=36, V=53, B=3)
    full = oracle.lm_head_gemv(t["hidden"], t["gamma"], t["lm_head"], eps=1e-4)
    want = np_normed(t["hidden"], t["gamma"], 1e-4) @ f64(t["lm_head"]).T
    assert full.shape == (3, 53)
    np.testing.assert_allclose(full, want, rtol=1e-11, atol=1e-12)
    rows = np.array([52, 0, 7, 7, 13], np.int32)
    assert np.array_equal(oracle.lm_head_rows(t["hidden"], t["gamma"], t["lm_head"], rows, eps=1e-4), full[:, rows])


def test_verification_is_argmax_membership(oracle):
    t = small(31, d=20, V=29, K=3, B=12)
    full = oracle.lm_head_gemv(t["hidden"], t["gamma"], t["lm_head"])
    # put the true arg-max among the ids for half of the tokens
    am = full.argmax(axis=1)
    t["ids"][::2, 1] = am[::2]
    for n in range(1, 12, 2):
        while am[n] in t["ids"][n]:
            t["ids"][n] = (t["ids"][n] + 1) % 29
    v = oracle.verify(t["hidden"], t["gamma"], t["lm_head"], t["ids"])
    assert np.array_equal(v["token"], am)
    assert np.array_equal(v["max_logit"], full.max(axis=1))
    assert v["hit"].tolist() == [1, 0] * 6


def test_verification_tie_goes_to_lowest_id(oracle):
    t = small(32, d=8, V=6, K=2, B=1)
    t["lm_head"][4] = t["lm_head"][2]
    t["lm_head"][2] = t["lm_head"][4] = (8 * np.sign(f64(t["hidden"][0]) * f64(t["gamma"]))).astype(np.float16)
    v = oracle.verify(t["hidden"], t["gamma"], t["lm_head"], np.array([[4, 5]], np.int32))
    assert v["token"][0] == 2 and v["hit"][0] == 0


# ---------------------------------------------------------------- early-exit loop down the layer stack
def loop_case(seed, L=6, B=5, d=24, V=23, K=3, H=16):
    rng = np.random.default_rng(seed)
    return dict(
        hidden=rng.standard_normal((L, B, d)).astype(np.float16),
        gamma=(1 + 0.1 * rng.standard_normal(d)).astype(np.float16),
        lm_head=(0.3 * rng.standard_normal((V, d))).astype(np.float16),
        ids=np.stack([rng.choice(V, K, replace=False) for _ in range(B)]).astype(np.int32),
        W1=(0.5 * rng.standard_normal((L, H, 3 * K))).astype(np.float16),
        w2=(0.5 * rng.standard_normal((L, H))).astype(np.float16),
        b1=(0.5 * rng.standard_normal((L, H))).astype(np.float16),
        b2=(0.5 * rng.standard_normal(L)).astype(np.float16))


def numpy_loop(t, threshold, active=None, eps=1e-5):
    """The decode loop written with numpy / scipy library routines only (float64)."""
    L, B, _ = t["hidden"].shape
    K = t["ids"].shape[1]
    W = f64(t["lm_head"])
    out = dict(scores=np.zeros((L, B)), exit=np.zeros((L, B), np.int32), ver_token=np.full((L, B), -1, np.int32),
               hit=np.zeros((L, B), np.int32), exit_layer=np.full(B, -1, np.int32), token=np.full(B, -1, np.int32),
               probs=np.zeros((L, B, K)))
    for b in range(B):
        prev = np.zeros(K, np.float32)
        for l in range(L):
            if active is not None and not active[l]:
                continue
            y = W @ np_normed(t["hidden"][l, b], t["gamma"], eps)        # every vocabulary logit
            z = y[t["ids"][b]]
            p = softmax(z)
            feat = np.concatenate([z, p, p - f64(prev)])
            a = np.maximum(f64(t["W1"][l]) @ feat + f64(t["b1"][l]), 0.0)
            s = expit(f64(t["w2"][l]) @ a + float(t["b2"][l]))
            out["scores"][l, b], out["probs"][l, b] = s, p
            prev = p.astype(np.float32)
            if np.float32(s) > np.float32(threshold):
                out["exit"][l, b] = 1
                tok = int(np.argmax(y))
                out["ver_token"][l, b] = tok
                if tok in t["ids"][b]:
                    out["hit"][l, b] = 1
                    out["exit_layer"][b], out["token"][b] = l, tok
                    break
    return out


def plant_hits(t, layers):
    """Token b's first id becomes the arg-max token of layer layers[b] (None: left alone)."""
    W = f64(t["lm_head"])
    for b, l in enumerate(layers):
        if l is None:
            continue
        tok = int(np.argmax(W @ np_normed(t["hidden"][l, b], t["gamma"], 1e-5)))
        others = [i for i in t["ids"][b] if i != tok][: t["ids"].shape[1] - 1]
        t["ids"][b] = [tok] + others
    return t


@pytest.mark.parametrize("threshold", [0.3, 0.5, -1.0])
def test_layer_loop_matches_numpy_decode_loop(oracle, threshold):
    t = plant_hits(loop_case(41), [4, 0, None, 2, 5])
    ref = numpy_loop(t, threshold)
    got = oracle.layer_loop(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"],
                            threshold=threshold)
    assert np.all(np.abs(ref["scores"][ref["scores"] != 0] - threshold) > 1e-6)
    for k in ("exit", "ver_token", "hit", "exit_layer", "token"):
        assert np.array_equal(got[k], ref[k]), k
    np.testing.assert_allclose(got["scores"], ref["scores"], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(got["probs"], ref["probs"], rtol=1e-9, atol=1e-12)
    if threshold < 0:       # every predictor fires: the exit layer is the first layer whose arg-max is speculative
        assert got["exit_layer"][1] == 0 and got["exit_layer"][3] <= 2 and got["exit_layer"][0] <= 4
        assert got["hit"].sum() == (got["exit_layer"] >= 0).sum() and (got["exit_layer"] >= 0).sum() >= 4


def test_layer_loop_that_never_fires_is_the_layer_sweep(oracle):
    t = plant_hits(loop_case(42), [1, 2, 3, 4, 5])
    got = oracle.layer_loop(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"],
                            threshold=2.0)
    sw = oracle.predict_sweep(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"],
                              threshold=2.0)
    for k in ("logits", "probs", "scores", "exit"):
        assert np.array_equal(got[k], sw[k]), k
    assert np.all(got["exit_layer"] == -1) and np.all(got["token"] == -1) and np.all(got["ver_token"] == -1)
    assert not got["hit"].any()


def test_layer_loop_nothing_is_evaluated_after_the_exit_or_on_inactive_layers(oracle):
    t = plant_hits(loop_case(43), [2, 2, 2, 2, 2])
    kw = dict(threshold=-1.0)
    a = (t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"])
    got = oracle.layer_loop(*a, **kw)
    assert np.all(got["exit_layer"] <= 2) and np.all(got["exit_layer"] >= 0)
    for b in range(5):
        e = got["exit_layer"][b]
        assert not got["scores"][e + 1:, b].any() and not got["probs"][e + 1:, b].any()
        assert np.all(got["ver_token"][e + 1:, b] == -1) and got["token"][b] == got["ver_token"][e, b]
    # with layers 0..2 inactive the planted layer cannot be used: same as the loop on the remaining layers
    active = np.array([0, 0, 0, 1, 1, 1], np.int32)
    got = oracle.layer_loop(*a, active=active, **kw)
    ref = numpy_loop(t, -1.0, active=active)
    assert not got["scores"][:3].any() and np.all(got["ver_token"][:3] == -1)
    for k in ("exit", "ver_token", "hit", "exit_layer", "token"):
        assert np.array_equal(got[k], ref[k]), k
    np.testing.assert_allclose(got["scores"], ref["scores"], rtol=1e-9, atol=1e-12)
    # the carried probabilities of a token come from its own previous *active* layer: zero before layer 3
    first = oracle.predict(t["hidden"][3], t["gamma"], t["lm_head"], t["ids"], np.zeros((5, 3), np.float32),
                           t["W1"][3], t["w2"][3], t["b1"][3], t["b2"][3:4], threshold=-1.0)
    assert np.array_equal(first["scores"], got["scores"][3])


def loop_case_q4(seed, L=6, B=5, d=32, V=23, K=3, H=16, group=16):
    """A decode-loop case on a quantised head whose weights fp16 holds exactly (power-of-two scales, integer
    zero-points), together with that fp16 head."""
    t = loop_case(seed, L=L, B=B, d=d, V=V, K=K, H=H)
    rng = np.random.default_rng(seed + 1000)
    codes = rng.integers(0, 16, size=(V, d)).astype(np.uint32)
    q = (codes.reshape(V, d // 8, 8) << (4 * np.arange(8, dtype=np.uint32))).sum(axis=2, dtype=np.uint32)
    scales = (2.0 ** rng.integers(-6, -2, size=(V, d // group))).astype(np.float16)
    zeros = rng.integers(0, 16, size=(V, d // group)).astype(np.float16)
    w = f64(scales).repeat(group, axis=1) * (codes.astype(np.float64) - f64(zeros).repeat(group, axis=1))
    w16 = w.astype(np.float16)
    assert np.array_equal(f64(w16), w)
    t["lm_head"] = w16
    return t, q, scales, zeros, group


@pytest.mark.parametrize("threshold", [0.4, -1.0])
def test_layer_loop_q4_is_the_pinned_loop_on_representable_weights(oracle, threshold):
    t, q, scales, zeros, group = loop_case_q4(51)
    t = plant_hits(t, [3, 0, None, 1, 5])
    got = oracle.layer_loop_q4(t["hidden"], t["gamma"], q, scales, zeros, group, t["ids"], t["W1"], t["w2"], t["b1"],
                               t["b2"], threshold=threshold)
    ref = oracle.layer_loop(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"],
                            threshold=threshold)
    lib = numpy_loop(t, threshold)
    assert np.all(np.abs(ref["scores"][ref["scores"] != 0] - threshold) > 1e-6)
    for k in ("exit", "ver_token", "hit", "exit_layer", "token"):
        assert np.array_equal(got[k], ref[k]), k
        assert np.array_equal(got[k], lib[k]), k
    for k in ("logits", "probs", "scores"):
        np.testing.assert_allclose(got[k], ref[k], rtol=1e-10, atol=1e-12)
    if threshold < 0:
        assert (got["exit_layer"] >= 0).sum() >= 3 and got["exit_layer"][1] == 0


def test_layer_loop_q4_that_never_fires_is_the_chain_of_quantised_predictors(oracle):
    t, codes, q, scales, zeros, group = q4_case(52, d=64, V=19, K=3, H=16, B=4, group=16)
    L, B = 5, 4
    lt = loop_case(52, L=L, B=B, d=64, V=19, K=3, H=16)
    active = np.array([1, 0, 1, 1, 0], np.int32)
    got = oracle.layer_loop_q4(lt["hidden"], lt["gamma"], q, scales, zeros, group, lt["ids"], lt["W1"], lt["w2"],
                               lt["b1"], lt["b2"], active=active, threshold=2.0)
    carry = np.zeros((B, 3), np.float32)
    for l in range(L):
        if not active[l]:
            assert not got["scores"][l].any() and not got["probs"][l].any()
            continue
        one = oracle.predict_q4(lt["hidden"][l], lt["gamma"], q, scales, zeros, group, lt["ids"], carry, lt["W1"][l],
                                lt["w2"][l], lt["b1"][l], lt["b2"][l:l + 1], threshold=2.0)
        for k in ("logits", "probs", "scores"):
            assert np.array_equal(got[k][l], one[k]), (k, l)
        carry = one["probs"].astype(np.float32)
    assert np.all(got["exit_layer"] == -1) and np.all(got["ver_token"] == -1) and not got["hit"].any()


# ---------------------------------------------------------------- online scheduling
def test_schedule_constant_exit_layer_closed_form(oracle):
    L, Q, e = 12, 5, 7
    active, counters = oracle.schedule(np.full(9, e, np.int32), L=L, Q=Q, radius=2)
    for t in range(9):
        want = np.zeros(L, int); want[e - 2:e + 3] = min(t, Q)
        assert np.array_equal(counters[t], want)
        assert np.array_equal(active[t], (want > 0).astype(int))


def test_schedule_queue_forgets_after_q_tokens_and_unions_offline_mask(oracle):
    L, Q = 16, 3
    seq = np.array([2, 2, 2, 12, 12, 12, 12], np.int32)
    off = np.zeros(L, np.int32); off[15] = 1
    active, counters = oracle.schedule(seq, L=L, Q=Q, radius=1, offline_mask=off)
    assert counters[3, 1:4].tolist() == [3, 3, 3] and counters[3, 11:14].tolist() == [0, 0, 0]
    assert counters[4, 1:4].tolist() == [2, 2, 2] and counters[4, 11:14].tolist() == [1, 1, 1]
    assert counters[6, 1:4].tolist() == [0, 0, 0] and counters[6, 11:14].tolist() == [3, 3, 3]
    assert np.all(active[:, 15] == 1) and active[0].sum() == 1
    assert active[6].tolist() == [0] * 11 + [1, 1, 1, 0, 1]
    # edges are clipped, not wrapped
    a2, c2 = oracle.schedule(np.array([0, 15], np.int32), L=L, Q=Q, radius=2)
    assert c2[1].tolist() == [1, 1, 1] + [0] * 13


def test_schedule_brute_force_random(oracle):
    rng = np.random.default_rng(5)
    L, Q, R, T = 32, 5, 2, 60
    seq = rng.integers(0, L, T).astype(np.int32)
    active, counters = oracle.schedule(seq, L=L, Q=Q, radius=R)
    for t, i in itertools.product(range(T), range(L)):
        last = seq[max(0, t - Q):t]
        assert counters[t, i] == int(np.sum(np.abs(last - i) <= R))
    assert np.array_equal(active, (counters > 0).astype(np.int32))


# ---------------------------------------------------------------- quantised LM-head rows (4-bit, per-group scale / zero)
def q4_case(seed, d=64, V=11, K=3, H=16, B=4, group=16):
    rng = np.random.default_rng(seed)
    t = small(seed, d=d, V=V, K=K, H=H, B=B)
    codes = rng.integers(0, 16, size=(V, d)).astype(np.uint32)
    q = (codes.reshape(V, d // 8, 8) << (4 * np.arange(8, dtype=np.uint32))).sum(axis=2, dtype=np.uint32)
    scales = (0.02 + 0.05 * rng.random((V, d // group))).astype(np.float16)
    zeros = rng.integers(0, 16, size=(V, d // group)).astype(np.float16)
    return t, codes, q, scales, zeros, group


def run_q4(oracle, t, q, scales, zeros, group, **kw):
    return oracle.predict_q4(t["hidden"], t["gamma"], q, scales, zeros, group, t["ids"], t["prev_probs"], t["W1"],
                             t["w2"], t["b1"], t["b2"], **kw)


def test_q4_unit_scale_zero_offset_is_the_fp16_predictor_on_the_codes(oracle):
    """scale 1, zero 0: the weights ARE the codes (0..15, exact in fp16), so every output must equal the
    already pinned fp16 predictor on a head that holds the codes."""
    t, codes, q, scales, zeros, group = q4_case(41)
    ones, nought = np.ones_like(scales), np.zeros_like(zeros)
    got = run_q4(oracle, t, q, ones, nought, group)
    ref = oracle.predict(t["hidden"], t["gamma"], codes.astype(np.float16), t["ids"], t["prev_probs"], t["W1"],
                         t["w2"], t["b1"], t["b2"])
    for k in ("logits", "probs", "features", "scores"):
        np.testing.assert_allclose(got[k], ref[k], rtol=1e-12, atol=1e-12)
    assert np.array_equal(got["exit"], ref["exit"])


def test_q4_equals_fp16_predictor_when_the_weights_are_representable(oracle):
    """Power-of-two scales and integer zero-points give weights that fp16 holds exactly: again the pinned
    fp16 predictor must agree, now with scale, zero-point and group index all in play."""
    t, codes, q, scales, zeros, group = q4_case(42, d=96, group=32)
    rng = np.random.default_rng(1)
    scales = (2.0 ** rng.integers(-6, -1, size=scales.shape)).astype(np.float16)
    w = f64(scales).repeat(group, axis=1) * (codes.astype(np.float64) - f64(zeros).repeat(group, axis=1))
    w16 = w.astype(np.float16)
    assert np.array_equal(f64(w16), w)
    got = run_q4(oracle, t, q, scales, zeros, group)
    ref = oracle.predict(t["hidden"], t["gamma"], w16, t["ids"], t["prev_probs"], t["W1"], t["w2"], t["b1"], t["b2"])
    np.testing.assert_allclose(got["logits"], ref["logits"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got["scores"], ref["scores"], rtol=1e-12, atol=1e-12)


def test_q4_nibble_order_and_group_index_one_hot(oracle):
    """A single non-zero code at element i (all zero-points 0) leaves logit = x_i * scale[group of i] * code:
    wrong nibble order, word index or group index each move it."""
    d, group, V = 64, 16, 3
    rng = np.random.default_rng(3)
    t = small(43, d=d, V=V, K=1, H=8, B=1)
    t["ids"][:] = 1
    x = np_normed(t["hidden"], t["gamma"], 1e-5)[0]
    scales = (0.5 + rng.random((V, d // group))).astype(np.float16)
    zeros = np.zeros((V, d // group), np.float16)
    for i in (0, 1, 7, 8, 15, 16, 37, 63):
        codes = np.zeros((V, d), np.uint32)
        codes[1, i] = 1 + i % 15
        q = (codes.reshape(V, d // 8, 8) << (4 * np.arange(8, dtype=np.uint32))).sum(axis=2, dtype=np.uint32)
        got = run_q4(oracle, t, q, scales, zeros, group)
        want = x[i] * float(scales[1, i // group]) * codes[1, i]
        assert math.isclose(got["logits"][0, 0], want, rel_tol=1e-12, abs_tol=1e-15), i


def test_q4_zero_point_shift_closed_form_and_dead_groups(oracle):
    t, codes, q, scales, zeros, group = q4_case(44, d=64, group=16)
    base = run_q4(oracle, t, q, scales, zeros, group)["logits"]
    # raising every zero-point by c lowers logit k by c * sum_g scale[id_k][g] * sum_{i in g} x_i
    x = np_normed(t["hidden"], t["gamma"], 1e-5)
    xg = x.reshape(x.shape[0], -1, group).sum(axis=2)                       # [B][groups]
    c = 3.0
    shifted = run_q4(oracle, t, q, scales, (f64(zeros) + c).astype(np.float16), group)["logits"]
    want = base - c * np.einsum("bg,bkg->bk", xg, f64(scales)[t["ids"]])
    np.testing.assert_allclose(shifted, want, rtol=1e-11, atol=1e-11)
    # a group whose scale is 0 contributes nothing, whatever its codes are
    s0 = scales.copy(); s0[:, 2] = 0
    a = run_q4(oracle, t, q, s0, zeros, group)["logits"]
    codes2 = codes.copy(); codes2[:, 2 * group:3 * group] = 15 - codes2[:, 2 * group:3 * group]
    q2 = (codes2.reshape(codes.shape[0], -1, 8) << (4 * np.arange(8, dtype=np.uint32))).sum(axis=2, dtype=np.uint32)
    b = run_q4(oracle, t, q2, s0, zeros, group)["logits"]
    assert np.array_equal(a, b)
    assert not np.array_equal(a, base)


def test_q4_generator_reconstructs_within_half_a_step(oracle):
    """The synthetic quantiser (input preparation) and the oracle's reading of the format agree: the weights
    the oracle sees differ from the fp16 originals by at most half a quantisation step per element, hence the
    logits by a bound that follows from it."""
    rng = np.random.default_rng(9)
    d, V, group = 256, 7, 128
    w = (0.02 * rng.standard_normal((V, d))).astype(np.float16)
    q, scales, zeros = synth.quantize_q4(w, group)
    assert q.dtype == np.uint32 and q.shape == (V, d // 8) and scales.shape == (V, d // group)
    t = small(45, d=d, V=V, K=2, H=8, B=3)
    got = run_q4(oracle, t, q, scales, zeros, group)["logits"]
    ref = oracle.predict(t["hidden"], t["gamma"], w, t["ids"], t["prev_probs"], t["W1"], t["w2"], t["b1"],
                         t["b2"])["logits"]
    x = np.abs(np_normed(t["hidden"], t["gamma"], 1e-5)).reshape(3, -1, group).sum(axis=2)      # [B][groups]
    bound = 0.5 * 1.01 * np.einsum("bg,bkg->bk", x, f64(scales)[t["ids"]]) + 1e-9
    assert np.all(np.abs(got - ref) <= bound)
    assert np.abs(got - ref).max() > 0


def test_q4_rejects_bad_arguments(oracle):
    t, codes, q, scales, zeros, group = q4_case(46)
    with pytest.raises(ValueError):
        run_q4(oracle, dict(t, ids=np.full_like(t["ids"], 11)), q, scales, zeros, group)
    t2, _, q2, _, _, _ = q4_case(47, d=48, group=8)
    s12 = np.ones((q2.shape[0], 4), np.float16)
    with pytest.raises(ValueError):                     # group must be a multiple of 8
        run_q4(oracle, t2, q2, s12, s12, 12)


# ---------------------------------------------------------------- full head, verification and tree on the quantised head
def np_dequant(codes, scales, zeros, group):
    return f64(scales).repeat(group, axis=1) * (codes.astype(np.float64) - f64(zeros).repeat(group, axis=1))


def test_q4_full_head_matches_numpy_matmul_on_dequantised_weights_and_the_predictor_rows(oracle):
    t, codes, q, scales, zeros, group = q4_case(51, d=96, V=29, K=3, B=5, group=32)
    full = oracle.lm_head_gemv_q4(t["hidden"], t["gamma"], q, scales, zeros, group)
    want = np_normed(t["hidden"], t["gamma"], 1e-5) @ np_dequant(codes, scales, zeros, group).T
    np.testing.assert_allclose(full, want, rtol=1e-11, atol=1e-11)
    # the reduced logits of the quantised predictor are these logits at the ids (same routine: bit-equal)
    pred = run_q4(oracle, t, q, scales, zeros, group)
    assert np.array_equal(pred["logits"], np.take_along_axis(full, t["ids"], axis=1))
    # weights that fp16 holds exactly: the pinned fp16 head on them
    rng = np.random.default_rng(2)
    s2 = (2.0 ** rng.integers(-6, -1, size=scales.shape)).astype(np.float16)
    w16 = np_dequant(codes, s2, zeros, group).astype(np.float16)
    assert np.array_equal(f64(w16), np_dequant(codes, s2, zeros, group))
    np.testing.assert_allclose(oracle.lm_head_gemv_q4(t["hidden"], t["gamma"], q, s2, zeros, group),
                               oracle.lm_head_gemv(t["hidden"], t["gamma"], w16), rtol=1e-12, atol=1e-12)


def test_q4_verification_is_argmax_membership_on_the_dequantised_head(oracle):
    t, codes, q, scales, zeros, group = q4_case(52, d=64, V=31, K=3, B=12, group=16)
    want = np_normed(t["hidden"], t["gamma"], 1e-5) @ np_dequant(codes, scales, zeros, group).T
    am = want.argmax(axis=1)
    t["ids"][::2, 1] = am[::2]
    for n in range(1, 12, 2):
        while am[n] in t["ids"][n]:
            t["ids"][n] = (t["ids"][n] + 1) % 31
    v = oracle.verify_q4(t["hidden"], t["gamma"], q, scales, zeros, group, t["ids"])
    assert np.array_equal(v["token"], am)
    np.testing.assert_allclose(v["max_logit"], want.max(axis=1), rtol=1e-11, atol=1e-11)
    assert v["hit"].tolist() == [1, 0] * 6
    # two identical quantised rows: the lower id wins
    codes[20] = codes[int(am[0])]
    scales[20], zeros[20] = scales[int(am[0])], zeros[int(am[0])]
    q2 = (codes.reshape(31, -1, 8) << (4 * np.arange(8, dtype=np.uint32))).sum(axis=2, dtype=np.uint32)
    v2 = oracle.verify_q4(t["hidden"][:1], t["gamma"], q2, scales, zeros, group, t["ids"][:1])
    assert v2["token"][0] == min(20, int(am[0]))


def test_q4_tree_equals_independent_quantised_predictors_and_the_fp16_tree_on_representable_weights(oracle):
    rng = np.random.default_rng(53)
    d, V, K, H, N, G, group = 64, 23, 3, 16, 9, 2, 16
    t, codes, q, scales, zeros, _ = q4_case(53, d=d, V=V, K=K, H=H, B=N, group=group)
    hidden = rng.standard_normal((G, N, d)).astype(np.float16)
    ids = rng.integers(0, V, size=(G, N, K)).astype(np.int32)
    prev = rng.dirichlet(np.ones(K), size=(G, N)).astype(np.float32)
    parent = np.tile(np.array([-1, 0, 0, 1, 1, 2, 3, 3, 5], np.int32), (G, 1))
    tree = oracle.predict_tree_q4(hidden, t["gamma"], q, scales, zeros, group, ids, prev, t["W1"], t["w2"], t["b1"],
                                  t["b2"], parent=parent, Mcap=27)
    for g in range(G):
        u, inv = np.unique(ids[g], return_inverse=True)
        assert tree["M"][g] == len(u) and np.array_equal(tree["merged"][g][:len(u)], u)
        assert np.all(tree["merged"][g][len(u):] == -1) and np.array_equal(tree["cols"][g].ravel(), inv.ravel())
        one = oracle.predict_q4(hidden[g], t["gamma"], q, scales, zeros, group, ids[g], prev[g], t["W1"], t["w2"],
                                t["b1"], t["b2"])
        for k in ("logits", "probs", "scores", "exit"):
            assert np.array_equal(tree[k][g], one[k]), k
        for n in range(N):                       # the path rule by walking to the root
            ok, cur = 1, n
            while cur >= 0:
                ok &= int(one["exit"][cur])
                cur = int(parent[g, cur])
            assert tree["path_exit"][g, n] == ok
    assert 0 < tree["exit"].sum() < tree["exit"].size
    s2 = (2.0 ** rng.integers(-6, -1, size=scales.shape)).astype(np.float16)
    w16 = np_dequant(codes, s2, zeros, group).astype(np.float16)
    a = oracle.predict_tree_q4(hidden, t["gamma"], q, s2, zeros, group, ids, prev, t["W1"], t["w2"], t["b1"], t["b2"],
                               parent=parent, Mcap=27)
    b = oracle.predict_tree(hidden, t["gamma"], w16, ids, prev, t["W1"], t["w2"], t["b1"], t["b2"], parent=parent,
                            Mcap=27)
    np.testing.assert_allclose(a["logits"], b["logits"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a["scores"], b["scores"], rtol=1e-12, atol=1e-12)
    assert np.array_equal(a["path_exit"], b["path_exit"]) and np.array_equal(a["cols"], b["cols"])
    with pytest.raises(ValueError):              # merged set larger than the capacity
        oracle.predict_tree_q4(hidden, t["gamma"], q, scales, zeros, group, ids, prev, t["W1"], t["w2"], parent=parent,
                               Mcap=3)
