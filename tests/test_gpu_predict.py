"""GPU parity: specee_predict / specee_predict_sweep / lm_head_gemv against the CPU oracle,
element by element on the same seeded inputs, through the C ABI."""
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
    assert torch.cuda.is_available()
    return specee


_LM = {}


def lm_for(c):
    key = (c.V, c.d)
    if key not in _LM:
        h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
        _LM[key] = (h, dev(h))
    return _LM[key]


def run_predict(sp, t, lm_d, **kw):
    out = sp.predict(dev(t["hidden"]), dev(t["gamma"]), lm_d, dev(t["ids"]), dev(t["prev_probs"]), dev(t["W1"]),
                     dev(t["w2"]), dev(t["b1"]), dev(t["b2"]), **kw)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in out.items()}


def custom(seed, d, V, K, H, B, bias):
    rng = np.random.default_rng(seed)
    return dict(
        hidden=rng.standard_normal((B, d)).astype(np.float16),
        gamma=(1 + 0.05 * rng.standard_normal(d)).astype(np.float16),
        lm_head=(0.05 * rng.standard_normal((V, d))).astype(np.float16),
        ids=np.stack([rng.choice(V, K, replace=False) for _ in range(B)]).astype(np.int32),
        prev_probs=rng.dirichlet(np.ones(K), size=B).astype(np.float32),
        W1=(0.1 * rng.standard_normal((H, 3 * K))).astype(np.float16),
        w2=(0.1 * rng.standard_normal(H)).astype(np.float16),
        b1=(0.1 * rng.standard_normal(H)).astype(np.float16) if bias else None,
        b2=(0.1 * rng.standard_normal(1)).astype(np.float16) if bias else None)


@pytest.mark.parametrize("d,V,K,H,B,bias", [
    (8, 5, 1, 1, 1, False),            # smallest legal shape
    (64, 50, 3, 40, 5, True),          # K not a power of two
    (1032, 301, 4, 512, 7, False),     # ragged d (129 vectors)
    (4104, 97, 4, 513, 3, True),       # d just over one 512-thread tile, H just over one pass
    (8192, 211, 8, 512, 4, False),     # two vectors per thread, K = 8
    (16384, 64, 8, 1024, 2, True),     # largest d, four vectors per thread
    (12296, 33, 16, 2048, 2, True),    # K = KMAX, H = HMAX, ragged tail beyond the unrolled tiles
    (2048, 500, 12, 100, 9, False),    # K between specialisations
    (520, 77, 5, 7, 33, True),
    (4096, 1000, 2, 512, 6, False),
])
def test_predict_shapes(sp, oracle, d, V, K, H, B, bias):
    t = custom(d * 7 + K, d, V, K, H, B, bias)
    ref = oracle.predict(**t, eps=1e-5, threshold=0.5)
    got = run_predict(sp, t, dev(t["lm_head"]))
    check_scored(got, ref, 0.5, f"d={d} K={K} H={H}")


def test_predict_c1_llama7b_shape(sp, oracle):
    c = synth.CONFIGS["C1"]
    lm_h, lm_d = lm_for(c)
    worst = {}
    exits = 0
    for seed in range(8):
        t = synth.make("C1", seed=seed, lm=lm_h)
        ref = oracle.predict(t["hidden"], t["gamma"], lm_h, t["ids"], t["prev_probs"], t["W1"], t["w2"],
                             eps=c.eps, threshold=c.threshold)
        got = run_predict(sp, t, lm_d, eps=c.eps, threshold=c.threshold)
        e = check_scored(got, ref, c.threshold, f"C1 seed {seed}")
        exits += int(ref["exit"].sum())
        for k, v in e.items():
            worst[k] = max(worst.get(k, 0), v)
    print("C1 worst relative errors", worst, "exits", exits, "of 8")
    assert 0 < exits < 8


@pytest.mark.parametrize("d,K,B,bias", [(8192, 4, 1100, True), (4096, 8, 1030, False), (2056, 4, 1500, True),
                                        (8192, 8, 1024, False)])
def test_predict_large_batch_shapes(sp, oracle, d, K, B, bias):
    """More than a thousand tokens per launch take the 256-thread shape where it exists (K in {4, 8}, two or
    four vectors per thread, two hidden units per thread); every path must agree with the oracle, with done
    flags and with an invalid id."""
    t = custom(d + K + B, d, 700, K, 512, B, bias)
    lm_d = dev(t["lm_head"])
    got = run_predict(sp, t, lm_d)
    pick = np.array([0, 1, 255, 256, 1023, B - 1])
    sub = dict(t, hidden=t["hidden"][pick], ids=t["ids"][pick], prev_probs=t["prev_probs"][pick])
    check_scored({k: v[pick] for k, v in got.items()}, oracle.predict(**sub, eps=1e-5, threshold=0.5), 0.5,
                 f"large batch d={d} K={K}")
    assert np.all(np.isfinite(got["scores"]))
    done = (np.arange(B) % 5 == 0).astype(np.int32)
    bad = dict(t, ids=t["ids"].copy())
    bad["ids"][7, K - 1] = 700
    got_d = run_predict(sp, bad, lm_d, done=dev(done))
    on = done == 0
    on[7] = False
    for k in ("logits", "probs", "scores", "exit"):
        assert np.array_equal(got_d[k][on], got[k][on]), k
    assert np.all(got_d["scores"][done != 0] == 0) and np.isnan(got_d["scores"][7])
    assert np.array_equal(got_d["probs"][done != 0], t["prev_probs"][done != 0])


def test_predict_throughput_configuration_sampled_tokens(sp, oracle):
    """The batched launch the benchmark times (8000 tokens, ids distinct across the batch): every output of
    a sample of tokens against the oracle, and cheap whole-batch properties."""
    c = synth.CONFIGS["C1"]
    lm_h, lm_d = lm_for(c)
    B = 8000
    rng = np.random.default_rng(8000)
    hid = rng.standard_normal((B, c.d), dtype=np.float32).astype(np.float16)
    ids = rng.permutation(c.V)[:B * c.K].reshape(B, c.K).astype(np.int32)
    t = synth.make("C1", lm=lm_h)
    t = dict(t, hidden=hid, ids=ids, prev_probs=synth.prob_rows(B, c.K, 9))
    got = run_predict(sp, t, lm_d)
    pick = np.unique(np.concatenate([[0, B - 1], rng.integers(0, B, 96)]))
    ref = oracle.predict(hid[pick], t["gamma"], lm_h, ids[pick], t["prev_probs"][pick], t["W1"], t["w2"])
    check_scored({k: v[pick] for k, v in got.items()}, ref, c.threshold, "B=8000 sampled")
    np.testing.assert_allclose(got["probs"].sum(axis=1), 1.0, atol=1e-5)
    assert np.all(np.isfinite(got["scores"])) and 0.05 < got["exit"].mean() < 0.95


def test_predict_is_deterministic(sp):
    c = synth.CONFIGS["C1"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C1", seed=3, lm=lm_h)
    a = run_predict(sp, t, lm_d)
    b = run_predict(sp, t, lm_d)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_predict_reduced_logits_equal_full_head_at_ids(sp, oracle):
    """Invariant: speculative logits == full-vocabulary logits at the speculative ids (two different kernels)."""
    c = synth.CONFIGS["C1"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C1", seed=5, lm=lm_h)
    got = run_predict(sp, t, lm_d)
    full = host(sp.lm_head_gemv(dev(t["hidden"]), dev(t["gamma"]), lm_d))
    close(got["logits"][0], full[0, t["ids"][0]], 1.0, "reduced vs full")


def test_predict_invalid_id_gives_nan_and_no_exit(sp):
    t = custom(1, 256, 40, 4, 64, 3, False)
    t["ids"][1, 2] = 40          # == V
    t["ids"][2, 0] = -7
    got = run_predict(sp, t, dev(t["lm_head"]))
    assert np.all(np.isfinite(got["logits"][0])) and np.isfinite(got["scores"][0])
    for n in (1, 2):
        assert np.all(np.isnan(got["logits"][n])) and np.all(np.isnan(got["probs"][n]))
        assert np.isnan(got["scores"][n]) and got["exit"][n] == 0


def test_predict_zero_weights_strict_threshold(sp):
    t = custom(2, 512, 40, 4, 512, 4, False)
    t["W1"][:] = 0
    t["w2"][:] = 0
    got = run_predict(sp, t, dev(t["lm_head"]), threshold=0.5)
    assert np.array_equal(got["scores"], np.full(4, 0.5, np.float32)) and got["exit"].sum() == 0
    got = run_predict(sp, t, dev(t["lm_head"]), threshold=0.25)
    assert got["exit"].sum() == 4


def test_predict_empty_batch_and_argument_errors(sp):
    t = custom(3, 64, 20, 4, 16, 2, False)
    d_ = {k: dev(v) for k, v in t.items()}
    out = sp.predict(d_["hidden"][:0], d_["gamma"], d_["lm_head"], d_["ids"][:0], d_["prev_probs"][:0], d_["W1"],
                     d_["w2"])
    assert out["scores"].numel() == 0
    with pytest.raises(sp.SpeceeError) as ei:        # d not a multiple of 8
        sp.predict(d_["hidden"][:, :60].contiguous(), d_["gamma"][:60].contiguous(),
                   d_["lm_head"][:, :60].contiguous(), d_["ids"], d_["prev_probs"], d_["W1"], d_["w2"])
    assert ei.value.code == -1
    with pytest.raises(sp.SpeceeError) as ei:        # misaligned hidden pointer
        flat = torch.zeros(2 * 64 + 8, dtype=torch.float16, device="cuda")
        sp.predict(flat[4:4 + 128].view(2, 64), d_["gamma"], d_["lm_head"], d_["ids"], d_["prev_probs"], d_["W1"],
                   d_["w2"])
    assert ei.value.code == -2
    with pytest.raises(sp.SpeceeError):              # probs aliasing prev_probs
        o = dict(logits=torch.empty_like(d_["prev_probs"]), probs=d_["prev_probs"],
                 scores=torch.empty(2, device="cuda"), exit=torch.empty(2, dtype=torch.int32, device="cuda"))
        sp.predict(d_["hidden"], d_["gamma"], d_["lm_head"], d_["ids"], d_["prev_probs"], d_["W1"], d_["w2"], out=o)


# ---------------------------------------------------------------- layer sweep
def run_sweep(sp, t, lm_d, active=None, prev0=None, **kw):
    out = sp.predict_sweep(dev(t["hidden"]), dev(t["gamma"]), lm_d, dev(t["ids"]), dev(t["W1"]), dev(t["w2"]),
                           dev(t["b1"]), dev(t["b2"]), prev0=dev(prev0), active=dev(active), **kw)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in out.items()}


def check_sweep(got, ref, thr, what):
    e = {}
    e["logits"] = close(got["logits"], ref["logits"], 1.0, what + " logits")
    e["probs"] = close(got["probs"], ref["probs"], 1e-3, what + " probs")
    e["scores"] = close(got["scores"], ref["scores"], 1e-3, what + " scores")
    decided = np.abs(ref["scores"] - thr) > 1e-4
    assert np.array_equal(got["exit"][decided], ref["exit"][decided]), what + " exit"
    # first_exit is unique only if no undecided layer precedes it
    for b in range(ref["first_exit"].shape[0]):
        col = decided[:, b]
        fe = ref["first_exit"][b]
        upto = fe if fe >= 0 else col.shape[0]
        if col[:upto + 1].all() if fe >= 0 else col.all():
            assert got["first_exit"][b] == fe, what + f" first_exit[{b}]"
    return e


@pytest.mark.parametrize("bias", [False, True])
def test_sweep_small(sp, oracle, bias):
    t = synth.make("T2", bias=bias)
    c = t["cfg"]
    ref = oracle.predict_sweep(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"])
    got = run_sweep(sp, t, dev(t["lm_head"]))
    check_sweep(got, ref, c.threshold, "T2 sweep")


def test_sweep_with_inactive_layers_and_initial_probs(sp, oracle):
    t = synth.make("T2")
    active = np.array([0, 1, 0, 0, 1], np.int32)
    prev0 = synth.prob_rows(7, 4, 99)
    ref = oracle.predict_sweep(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], prev0=prev0,
                               active=active)
    got = run_sweep(sp, t, dev(t["lm_head"]), active=active, prev0=prev0)
    check_sweep(got, ref, 0.5, "T2 masked sweep")
    assert not got["scores"][0].any() and not got["probs"][2].any() and not got["exit"][3].any()


def test_sweep_equals_chained_predict_calls_on_gpu(sp):
    """The one-launch sweep must reproduce the sequential per-layer use of specee_predict."""
    t = synth.make("T2")
    c = t["cfg"]
    lm_d = dev(t["lm_head"])
    sw = run_sweep(sp, t, lm_d)
    prev = np.zeros((c.B, c.K), np.float32)
    for l in range(c.L):
        tl = dict(t, hidden=t["hidden"][l], prev_probs=prev, W1=t["W1"][l], w2=t["w2"][l])
        one = run_predict(sp, tl, lm_d)
        assert np.array_equal(one["scores"], sw["scores"][l]) and np.array_equal(one["probs"], sw["probs"][l])
        prev = one["probs"]


def test_sweep_c2_llama7b_32_layers(sp, oracle):
    c = synth.CONFIGS["C2"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C2", lm=lm_h)
    ref = oracle.predict_sweep(t["hidden"], t["gamma"], lm_h, t["ids"], t["W1"], t["w2"])
    got = run_sweep(sp, t, lm_d)
    e = check_sweep(got, ref, c.threshold, "C2")
    print("C2 worst", e, "first_exit", ref["first_exit"], "scores", np.round(ref["scores"][:, 0], 3))
    # sequential per-layer calls (the decode-time usage) give the same numbers
    prev = np.zeros((1, c.K), np.float32)
    for l in range(c.L):
        tl = dict(t, hidden=t["hidden"][l], prev_probs=prev, W1=t["W1"][l], w2=t["w2"][l])
        one = run_predict(sp, tl, lm_d)
        close(one["scores"], ref["scores"][l], 1e-3, f"C2 layer {l}")
        prev = one["probs"]


def test_c2_as_the_benchmark_launches_it_graph_of_32_dependent_calls(sp, oracle):
    """The headline step: 32 dependent specee_predict launches, each reading the previous layer's probabilities
    from device memory, captured once in a HIP graph and replayed.  Every replay must match the oracle's sweep."""
    c = synth.CONFIGS["C2"]
    lm_h, lm_d = lm_for(c)
    gamma = None
    sets = []
    for r in range(2):  # two input sets, as the benchmark rotates over several
        hid_h = synth.hidden_drift(c.L, 1, c.d, 50_000 + r)
        ids_h = synth.ids_uniform_distinct(1, c.K, c.V, 60_000 + r)
        base = synth.make("C2", lm=lm_h)
        gamma = dev(base["gamma"])
        W1, w2 = dev(base["W1"]), dev(base["w2"])
        out = dict(logits=torch.empty((c.L, 1, c.K), device="cuda"), probs=torch.empty((c.L, 1, c.K), device="cuda"),
                   scores=torch.empty((c.L, 1), device="cuda"),
                   exit=torch.empty((c.L, 1), dtype=torch.int32, device="cuda"))
        ref = oracle.predict_sweep(hid_h, base["gamma"], lm_h, ids_h, base["W1"], base["w2"])
        sets.append((dev(hid_h), dev(ids_h), W1, w2, out, torch.zeros((1, c.K), device="cuda"), ref))

    def calls(r):
        hid, ids, W1, w2, out, zero, _ = sets[r]
        for l in range(c.L):
            o = dict(logits=out["logits"][l], probs=out["probs"][l], scores=out["scores"][l], exit=out["exit"][l])
            sp.predict(hid[l], gamma, lm_d, ids, zero if l == 0 else out["probs"][l - 1], W1[l], w2[l], out=o)

    graphs = []
    stream = torch.cuda.Stream()
    for r in range(2):
        with torch.cuda.stream(stream):
            calls(r)  # eager once: nothing lazy is left to happen under capture
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                calls(r)
        graphs.append(g)
    torch.cuda.synchronize()
    for rep in range(3):
        for r in range(2):
            out, ref = sets[r][4], sets[r][6]
            for v in out.values():
                v.zero_()  # eager work between replays; the graph must rewrite every output
            graphs[r].replay()
            torch.cuda.synchronize()
            got = {k: host(v) for k, v in out.items()}
            close(got["logits"], ref["logits"], 1.0, f"graph replay {rep} set {r} logits")
            close(got["probs"], ref["probs"], 1e-3, f"graph replay {rep} set {r} probs")
            close(got["scores"], ref["scores"], 1e-3, f"graph replay {rep} set {r} scores")
            near = np.abs(ref["scores"].astype(np.float64) - c.threshold) < 1e-4
            assert np.array_equal(got["exit"][~near], ref["exit"][~near])


def test_sweep_c4_llama13b_16_sequences_40_layers(sp, oracle):
    c = synth.CONFIGS["C4"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C4", lm=lm_h)
    oracle.set_threads(8)
    ref = oracle.predict_sweep(t["hidden"], t["gamma"], lm_h, t["ids"], t["W1"], t["w2"])
    oracle.set_threads(1)
    got = run_sweep(sp, t, lm_d)
    e = check_sweep(got, ref, c.threshold, "C4")
    n_exit = int(ref["exit"].sum())
    print("C4 worst", e, "exits", n_exit, "of", ref["exit"].size, "distinct ids", len(np.unique(t["ids"])))
    assert 0 < n_exit < ref["exit"].size


# ---------------------------------------------------------------- full-vocabulary head
@pytest.mark.parametrize("d,V,N", [(8, 1, 1), (64, 37, 3), (1032, 1000, 2), (4096, 4099, 1), (8200, 515, 2),
                                   (16384, 130, 2)])      # the largest accepted hidden size (64 KB of LDS for x)
def test_lm_head_small(sp, oracle, d, V, N):
    t = custom(d + V, d, V, 1, 1, N, False)
    ref = oracle.lm_head_gemv(t["hidden"], t["gamma"], t["lm_head"])
    got = host(sp.lm_head_gemv(dev(t["hidden"]), dev(t["gamma"]), dev(t["lm_head"])))
    close(got, ref, 1.0, f"lm_head d={d} V={V}")


def test_lm_head_llama7b_full_vocab(sp, oracle):
    c = synth.CONFIGS["C1"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C1", seed=1, lm=lm_h)
    oracle.set_threads(8)
    ref = oracle.lm_head_gemv(t["hidden"], t["gamma"], lm_h)
    oracle.set_threads(1)
    got = host(sp.lm_head_gemv(dev(t["hidden"]), dev(t["gamma"]), lm_d))
    w = close(got, ref, 1.0, "lm_head 32000x4096")
    print("lm_head 32000x4096 worst", w)
    assert int(got.argmax()) == int(ref.argmax())


# ---------------------------------------------------------------- device status word
def test_status_word_reports_invalid_ids_and_merge_overflow(sp):
    t = synth.make("T3")
    c = t["cfg"]
    a = dict(hidden=dev(t["hidden"]), gamma=dev(t["gamma"]), lm=dev(t["lm_head"]), prev=dev(t["prev_probs"]),
             W1=dev(t["W1"]), w2=dev(t["w2"]), parent=dev(t["parent"]))

    def tree(ids, Mcap):
        o = sp.predict_tree(a["hidden"], a["gamma"], a["lm"], dev(ids), a["prev"], a["W1"], a["w2"], parent=a["parent"],
                            Mcap=Mcap)
        w = sp.status_word(o["scores"], o["M"].reshape(1), Mcap)
        torch.cuda.synchronize()
        return int(host(w)[0])
    assert tree(t["ids"], c.Mcap) == 0
    bad = t["ids"].copy()
    bad[5, 1] = c.V
    assert tree(bad, c.Mcap) == 1                       # an id outside the vocabulary
    assert tree(t["ids"], len(np.unique(t["ids"])) - 1) == 3   # overflow (its scores are NaN as well)
    p = custom(9, 256, 100, 4, 64, 300, False)
    ids = p["ids"].copy()
    ids[250, 3] = -7
    o = sp.predict(dev(p["hidden"]), dev(p["gamma"]), dev(p["lm_head"]), dev(ids), dev(p["prev_probs"]), dev(p["W1"]),
                   dev(p["w2"]))
    w = sp.status_word(o["scores"])
    torch.cuda.synchronize()
    assert int(host(w)[0]) == 1
