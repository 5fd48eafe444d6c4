"""GPU parity: specee_predict_tree (merged mapping) and the multi-state full-vocabulary head
against the CPU oracle, through the C ABI."""
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
        _LM.clear()      # keep at most one large head resident
        h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
        _LM[key] = (h, dev(h))
    return _LM[key]


def run_tree(sp, t, lm_d, Mcap, parent="auto", **kw):
    par = t.get("parent") if isinstance(parent, str) else parent
    out = sp.predict_tree(dev(t["hidden"]), dev(t["gamma"]), lm_d, dev(t["ids"]), dev(t["prev_probs"]),
                          dev(t["W1"]), dev(t["w2"]), dev(t["b1"]), dev(t["b2"]), parent=dev(par), Mcap=Mcap, **kw)
    torch.cuda.synchronize()
    res = {k: host(v) for k, v in out.items() if k != "_workspace"}
    res["parent"] = None if par is None else np.asarray(par)
    return res


def path_and(flags, parent):
    """AND of per-node flags from every node up to its root (parents precede children); [N] or [G][N]."""
    ex = np.asarray(flags).astype(bool)
    ex2, par2 = np.atleast_2d(ex), np.atleast_2d(np.asarray(parent))
    out = np.zeros_like(ex2)
    rows = np.arange(ex2.shape[0])
    for n in range(ex2.shape[1]):
        p = par2[:, n]
        assert np.all(p < n)
        out[:, n] = ex2[:, n] & np.where(p >= 0, out[rows, np.maximum(p, 0)], True)
    return out.reshape(ex.shape)


def check_tree(got, ref, thr, what, min_compared=0.5):
    # integer outputs: bit-exact
    assert np.array_equal(got["M"], ref["M"]), what + " M"
    assert np.array_equal(got["merged"], ref["merged"]), what + " merged ids"
    assert np.array_equal(got["cols"], ref["cols"]), what + " cols"
    e = check_scored(got, ref, thr, what)
    if ref.get("path_exit") is not None:
        parent = got["parent"]          # what run_tree passed to the library
        # the path rule applied to the GPU's own exit flags: every node, no exemption
        assert np.array_equal(got["path_exit"], path_and(got["exit"], parent).astype(np.int32)), \
            what + " path_exit is not the AND of the exit flags up to the root"
        # against the oracle: every node whose whole root path lies outside the band around the threshold
        decided = path_and(np.abs(ref["scores"] - thr) > 1e-4, parent)
        assert decided.mean() >= min_compared, (what, "too few nodes have a decided root path", decided.mean())
        assert np.array_equal(got["path_exit"][decided], ref["path_exit"][decided]), what + " path_exit"
    return e


def ref_tree(oracle, t, Mcap, **kw):
    return oracle.predict_tree(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["prev_probs"], t["W1"], t["w2"],
                               t["b1"], t["b2"], parent=t.get("parent"), Mcap=Mcap, **kw)


@pytest.mark.parametrize("name,bias", [("T3", False), ("T4", True)])
def test_tree_small(sp, oracle, name, bias):
    t = synth.make(name, bias=bias)
    c = t["cfg"]
    ref = ref_tree(oracle, t, c.Mcap)
    got = run_tree(sp, t, dev(t["lm_head"]), c.Mcap)
    e = check_tree(got, ref, c.threshold, name)
    print(name, "M", ref["M"], "worst", e)


def test_tree_equals_independent_predict_calls_on_gpu(sp):
    """Merged mapping == N independent per-node predictors (two different GPU code paths)."""
    t = synth.make("T3")
    c = t["cfg"]
    lm_d = dev(t["lm_head"])
    tree = run_tree(sp, t, lm_d, c.Mcap)
    ind = sp.predict(dev(t["hidden"]), dev(t["gamma"]), lm_d, dev(t["ids"]), dev(t["prev_probs"]), dev(t["W1"]),
                     dev(t["w2"]))
    torch.cuda.synchronize()
    close(tree["logits"], host(ind["logits"]), 1.0, "tree vs independent logits")
    close(tree["scores"], host(ind["scores"]), 1e-3, "tree vs independent scores")


def test_tree_and_predict_agree_on_hidden_states_with_large_outliers(sp, oracle):
    """A few hidden elements in the thousands (the outlier channels of real models): the matrix-core paths form
    h * gamma in fp16 before splitting it exactly, which holds up to 65504; merged tree, independent predictors
    and oracle must still agree."""
    t = make_tree(21, 1024, 500, 4, 512, 40)
    rng = np.random.default_rng(5)
    h = t["hidden"].astype(np.float32)
    for n in range(40):
        h[n, rng.integers(0, 1024, 3)] = rng.choice([-1.0, 1.0], 3) * rng.uniform(500, 3000, 3)
    t["hidden"] = h.astype(np.float16)
    t["gamma"] = (1.5 + 0.05 * rng.standard_normal(1024)).astype(np.float16)
    pool = rng.permutation(500)[:60]
    t["ids"] = pool[rng.integers(0, 60, size=(40, 4))].astype(np.int32)
    ref = ref_tree(oracle, t, 64)
    lm_d = dev(t["lm_head"])
    got = run_tree(sp, t, lm_d, 64)
    check_tree(got, ref, 0.5, "outlier hidden states", min_compared=0.3)
    ind = sp.predict(dev(t["hidden"]), dev(t["gamma"]), lm_d, dev(t["ids"]), dev(t["prev_probs"]), dev(t["W1"]),
                     dev(t["w2"]))
    torch.cuda.synchronize()
    close(host(ind["logits"]), ref["logits"], 1.0, "independent predictors, outlier hidden states")
    full = host(sp.lm_head_gemv(dev(t["hidden"][:8]), dev(t["gamma"]), lm_d))      # matrix-core head, same split
    close(full, oracle.lm_head_gemv(t["hidden"][:8], t["gamma"], t["lm_head"]), 1.0, "full head, outlier hidden states")


def make_tree(seed, d, V, K, H, N, ids=None, bias=False):
    rng = np.random.default_rng(seed)
    t = dict(
        hidden=rng.standard_normal((N, d)).astype(np.float16),
        gamma=(1 + 0.05 * rng.standard_normal(d)).astype(np.float16),
        lm_head=(0.05 * rng.standard_normal((V, d))).astype(np.float16),
        ids=ids if ids is not None else rng.integers(0, V, size=(N, K)).astype(np.int32),
        prev_probs=rng.dirichlet(np.ones(K), size=N).astype(np.float32),
        W1=(0.1 * rng.standard_normal((H, 3 * K))).astype(np.float16),
        w2=(0.1 * rng.standard_normal(H)).astype(np.float16),
        b1=(0.1 * rng.standard_normal(H)).astype(np.float16) if bias else None,
        b2=(0.1 * rng.standard_normal(1)).astype(np.float16) if bias else None,
        parent=np.array([-1] + [int(rng.integers(0, n)) for n in range(1, N)], np.int32))
    return t


def test_tree_all_nodes_share_ids_and_all_distinct(sp, oracle):
    same = np.tile(np.array([[17, 3, 250, 99]], np.int32), (20, 1))
    t = make_tree(1, 512, 300, 4, 64, 20, ids=same)
    ref = ref_tree(oracle, t, 16)
    assert ref["M"] == 4
    check_tree(run_tree(sp, t, dev(t["lm_head"]), 16), ref, 0.5, "shared ids")
    distinct = np.random.default_rng(2).permutation(300)[:80].reshape(20, 4).astype(np.int32)
    t = make_tree(3, 512, 300, 4, 64, 20, ids=distinct)
    ref = ref_tree(oracle, t, 80)
    assert ref["M"] == 80
    check_tree(run_tree(sp, t, dev(t["lm_head"]), 80), ref, 0.5, "distinct ids")


@pytest.mark.parametrize("d,V,K,H,N,Mcap", [
    (8, 9, 1, 1, 1, 1),              # smallest legal tree
    (64, 40, 2, 8, 100, 40),         # more than 64 nodes: two node blocks, duplicate ids inside a node allowed
    (520, 777, 8, 512, 21, 168),     # ragged d (not a multiple of 64)
    (4096, 2000, 4, 512, 60, 64),    # C3 shape on a small vocabulary, random (non-pooled) ids capped by V
    (1024, 5000, 16, 300, 50, 800),  # K = KMAX, several row groups
    (2048, 64, 3, 2048, 17, 51),     # K odd, H = HMAX
])
def test_tree_shapes(sp, oracle, d, V, K, H, N, Mcap):
    t = make_tree(d + N, d, V, K, H, N, bias=(K % 2 == 1))
    if len(np.unique(t["ids"])) > Mcap:
        pool = np.random.default_rng(0).permutation(V)[:Mcap]
        t["ids"] = pool[np.random.default_rng(1).integers(0, Mcap, size=(N, K))].astype(np.int32)
    ref = ref_tree(oracle, t, Mcap)
    check_tree(run_tree(sp, t, dev(t["lm_head"]), Mcap), ref, 0.5, f"tree d={d} K={K} N={N}")


def stack_trees(ts):
    stack = lambda k: np.stack([t[k] for t in ts])
    return dict(ts[0], hidden=stack("hidden"), ids=stack("ids"), prev_probs=stack("prev_probs"),
                parent=stack("parent"))


def test_tree_largest_supported_tree(sp, oracle):
    """N*K = 4096 ids (the documented limit): the stand-alone merge kernel at full size, eight node blocks,
    dozens of row groups, and the per-node finish (the per-tree finish would not fit in LDS)."""
    d, V, K, H, N = 64, 20000, 8, 64, 512
    t = make_tree(77, d, V, K, H, N)
    M = len(np.unique(t["ids"]))
    assert N * K == 4096 and M > 3000
    ref = ref_tree(oracle, t, 4096)
    got = run_tree(sp, t, dev(t["lm_head"]), 4096)
    check_tree(got, ref, 0.5, "4096-id tree")
    # a few of these in one call: the per-tree finish shape is skipped because its LDS need exceeds the limit
    tb = stack_trees([t, make_tree(78, d, V, K, H, N), make_tree(79, d, V, K, H, N)])
    for k in ("gamma", "lm_head", "W1", "w2", "b1", "b2"):
        tb[k] = t[k]
    ref = ref_tree(oracle, tb, 4096)
    got = run_tree(sp, tb, dev(tb["lm_head"]), 4096)
    check_tree(got, ref, 0.5, "three 4096-id trees")
    with pytest.raises(sp.SpeceeError):            # one node more than the limit
        big = make_tree(80, d, V, K, H, N + 1)
        run_tree(sp, big, dev(big["lm_head"]), 4096)


def test_tree_many_mid_size_trees_split_path(sp, oracle):
    """Forty trees with more than 64 nodes each: too wide for one workgroup per tree, so the d-split
    contraction runs with the stand-alone merge kernel and the per-tree finish (matrix-core MLP)."""
    d, V, K, H, N, Mcap = 256, 3000, 4, 512, 80, 200
    ts = []
    for gidx in range(40):
        t = make_tree(500 + gidx, d, V, K, H, N)
        pool = np.random.default_rng(gidx).permutation(V)[:Mcap]
        t["ids"] = pool[np.random.default_rng(900 + gidx).integers(0, Mcap, size=(N, K))].astype(np.int32)
        ts.append(t)
    for t in ts[1:]:
        for k in ("gamma", "lm_head", "W1", "w2", "b1", "b2"):
            t[k] = ts[0][k]
    tb = stack_trees(ts)
    ref = ref_tree(oracle, tb, Mcap)
    got = run_tree(sp, tb, dev(tb["lm_head"]), Mcap)
    check_tree(got, ref, 0.5, "40 trees of 80 nodes")


def test_tree_batch_of_independent_trees(sp, oracle):
    ts = [synth.make("T4", seed=s) for s in range(3)]
    c = ts[0]["cfg"]
    stack = lambda k: np.stack([t[k] for t in ts])
    tb = dict(ts[0], hidden=stack("hidden"), ids=stack("ids"), prev_probs=stack("prev_probs"), parent=stack("parent"))
    ref = ref_tree(oracle, tb, c.Mcap)
    got = run_tree(sp, tb, dev(tb["lm_head"]), c.Mcap)
    check_tree(got, ref, c.threshold, "batched trees")
    assert len(set(ref["M"].tolist())) > 1       # trees really differ in merged size


@pytest.mark.parametrize("name,G,bias", [("T3", 20, True), ("T3", 16, False), ("T3", 40, False), ("T3", 130, True),
                                         ("T3", 260, False)])
def test_tree_many_trees_one_workgroup_each(sp, oracle, name, G, bias):
    """Batches of small trees: below about twenty trees every tree is spread over the GPU; from there on
    a single launch does merge, contraction, scoring and path rule -- with a few workgroups per tree
    that hand their d-slices to the last one (20, 40 trees), one 512-thread workgroup per tree (130) or
    one 256-thread workgroup per tree (260).  All must agree with the oracle."""
    ts = [synth.make(name, seed=s, bias=bias) for s in range(G)]
    c = ts[0]["cfg"]
    tb = stack_trees(ts)
    ref = ref_tree(oracle, tb, c.Mcap)
    got = run_tree(sp, tb, dev(tb["lm_head"]), c.Mcap)
    check_tree(got, ref, c.threshold, f"{G} x {name}")
    assert 0 < ref["path_exit"].sum() < ref["exit"].sum()


@pytest.mark.parametrize("d,V,K,H,N,Mcap", [
    (520, 777, 8, 512, 21, 128),     # ragged d, K = 8, wide merged set (two row tiles per wave)
    (1024, 300, 3, 100, 64, 64),     # K odd (generic MLP path), full 64 nodes
    (256, 5000, 16, 2048, 40, 128),  # K = KMAX, H = HMAX
    (4096, 2000, 4, 512, 60, 64),    # C3 shape
    (64, 40, 1, 8, 5, 7),            # tiny
])
@pytest.mark.parametrize("G", [17, 33])
def test_tree_many_trees_shapes(sp, oracle, d, V, K, H, N, Mcap, G):
    ts = []
    for gidx in range(G):
        t = make_tree(1000 * gidx + d, d, V, K, H, N, bias=(K % 2 == 1))
        pool = np.random.default_rng(gidx).permutation(V)[:Mcap]
        t["ids"] = pool[np.random.default_rng(100 + gidx).integers(0, Mcap, size=(N, K))].astype(np.int32)
        ts.append(t)
    for t in ts[1:]:                 # one model: shared head, norm weight and predictor
        for k in ("gamma", "lm_head", "W1", "w2", "b1", "b2"):
            t[k] = ts[0][k]
    tb = stack_trees(ts)
    ref = ref_tree(oracle, tb, Mcap)
    got = run_tree(sp, tb, dev(tb["lm_head"]), Mcap)
    check_tree(got, ref, 0.5, f"{G} trees d={d} K={K} N={N}")


@pytest.mark.parametrize("d,V,K,H,N,Mcap,G", [
    (520, 777, 8, 512, 64, 256, 33),     # 129..256 merged rows: sixteen row tiles, seven d-slices per tree by ticket
    (520, 777, 8, 512, 64, 256, 130),    # one d-slice
    (520, 777, 8, 512, 61, 256, 260),    # more trees than CUs, ragged node count
    (1032, 900, 4, 512, 60, 200, 40),    # K = 4, capacity not a multiple of 16
    (8192, 700, 8, 512, 64, 256, 24),    # the large-vocabulary tree shape's d, eight d-slices of 1024
    (256, 5000, 16, 1024, 16, 256, 21),  # K = KMAX: every node fills the capacity on its own
])
def test_tree_many_trees_wide_merged_sets(sp, oracle, d, V, K, H, N, Mcap, G):
    ts = []
    for gidx in range(G):
        t = make_tree(77 * gidx + d, d, V, K, H, N, bias=True)
        # merged sets of different sizes within the capacity (each size class takes its own version of the
        # kernel's stage loop; the smallest leaves the upper row tiles empty)
        width = [Mcap, min(Mcap, 180), min(Mcap, 150), 90][gidx % 4]
        pool = np.random.default_rng(gidx).permutation(V)[:width]
        t["ids"] = pool[np.random.default_rng(300 + gidx).integers(0, width, size=(N, K))].astype(np.int32)
        ts.append(t)
    for t in ts[1:]:
        for k in ("gamma", "lm_head", "W1", "w2", "b1", "b2"):
            t[k] = ts[0][k]
    tb = stack_trees(ts)
    ref = ref_tree(oracle, tb, Mcap)
    assert ref["M"].max() > 128 or N * K <= 128
    if N * K >= 512 and Mcap == 256:
        ms = ref["M"]
        assert (ms > 192).any() and ((ms > 160) & (ms <= 192)).any() and ((ms > 128) & (ms <= 160)).any() and (ms <= 128).any()
    got = run_tree(sp, tb, dev(tb["lm_head"]), Mcap)
    check_tree(got, ref, 0.5, f"{G} trees d={d} K={K} N={N} Mcap={Mcap}")


@pytest.mark.parametrize("d,V,K,H,N,Mcap,G", [
    (1032, 900, 4, 512, 60, 64, 300),    # the 60-node, 64-row shape: matrix-core MLP from the padded predictor image
    (2048, 900, 8, 512, 30, 64, 300),    # K = 8
    (520, 777, 3, 100, 64, 48, 270),     # K odd: vector-unit MLP; ragged d
    (4096, 600, 4, 512, 60, 64, 520),    # full hidden size, two workgroups per CU and more than one round
])
def test_tree_more_trees_than_cus_narrow_merged_sets(sp, oracle, d, V, K, H, N, Mcap, G):
    """More than 256 trees with at most 64 merged rows each: one 256-thread workgroup per tree with four
    row tiles (below 257 trees the same shape takes 512 threads per tree)."""
    ts = []
    for gidx in range(G):
        t = make_tree(31 * gidx + d, d, V, K, H, N, bias=(gidx == 0 and K == 8))
        width = [Mcap, Mcap - 7, 33, 16][gidx % 4]
        pool = np.random.default_rng(gidx).permutation(V)[:width]
        t["ids"] = pool[np.random.default_rng(700 + gidx).integers(0, width, size=(N, K))].astype(np.int32)
        ts.append(t)
    for t in ts[1:]:
        for k in ("gamma", "lm_head", "W1", "w2", "b1", "b2"):
            t[k] = ts[0][k]
    tb = stack_trees(ts)
    oracle.set_threads(8)
    ref = ref_tree(oracle, tb, Mcap)
    oracle.set_threads(1)
    got = run_tree(sp, tb, dev(tb["lm_head"]), Mcap)
    check_tree(got, ref, 0.5, f"{G} trees d={d} K={K} N={N} Mcap={Mcap}")
    assert 0 < ref["path_exit"].sum() < ref["exit"].sum()


@pytest.mark.parametrize("G", [16, 24])
def test_tree_many_trees_overflow_invalid_ids_and_no_parent(sp, oracle, G):
    ts = [synth.make("T3", seed=s) for s in range(G)]
    c = ts[0]["cfg"]
    tb = stack_trees(ts)
    lm_d = dev(tb["lm_head"])
    Ms = [len(np.unique(t["ids"])) for t in ts]
    cap = sorted(Ms)[len(Ms) // 2]                       # about half of the trees overflow this capacity
    got = run_tree(sp, tb, lm_d, cap)
    assert np.array_equal(got["M"], np.array(Ms))
    over = np.array(Ms) > cap
    assert over.any() and not over.all()
    assert np.all(np.isnan(got["scores"][over])) and got["exit"][over].sum() == 0 and got["path_exit"][over].sum() == 0
    ref = ref_tree(oracle, tb, c.Mcap)
    close(got["scores"][~over], ref["scores"][~over], 1e-3, "trees that fit beside trees that overflow")
    bad = dict(tb, ids=tb["ids"].copy())
    bad["ids"][3, 4, 1] = c.V
    bad["ids"][7, 0, 0] = -3
    got = run_tree(sp, bad, lm_d, c.Mcap, parent=None)
    assert got["path_exit"] is None
    assert np.isnan(got["scores"][3, 4]) and np.isnan(got["scores"][7, 0]) and got["exit"][3, 4] == 0
    mask = np.ones((G, c.N), bool); mask[3, 4] = mask[7, 0] = False
    close(got["scores"][mask], ref["scores"][mask], 1e-3, "valid nodes beside invalid ones")


def test_tree_many_trees_c3_batch(sp, oracle):
    c = synth.CONFIGS["C3"]
    lm_h, lm_d = lm_for(c)
    ts = [synth.make("C3", seed=100 + s, lm=lm_h) for s in range(24)]
    tb = stack_trees(ts)
    oracle.set_threads(8)
    ref = ref_tree(oracle, tb, c.Mcap)
    oracle.set_threads(1)
    got = run_tree(sp, tb, lm_d, c.Mcap)
    e = check_tree(got, ref, c.threshold, "24 x C3")
    print("24 x C3 worst", e)
    one = dict(ts[0], hidden=ts[5]["hidden"], ids=ts[5]["ids"], prev_probs=ts[5]["prev_probs"], parent=ts[5]["parent"])
    single = run_tree(sp, one, lm_d, c.Mcap)            # the few-trees path gives the same answers
    close(got["scores"][5], single["scores"], 1e-3, "whole-tree vs split path")
    assert np.array_equal(got["merged"][5], single["merged"]) and np.array_equal(got["cols"][5], single["cols"])


@pytest.mark.parametrize("G", [24, 64, 100])
def test_tree_sliced_batch_is_reproducible(sp, G):
    """With a few workgroups per tree (eight, four, two here), whichever finishes last adds the d-slices up
    -- in slice order, so repeated launches give identical bits."""
    c = synth.CONFIGS["C3"]
    lm_h, lm_d = lm_for(c)
    ts = [synth.make("C3", seed=300 + s, lm=lm_h) for s in range(G)]
    tb = stack_trees(ts)
    first = run_tree(sp, tb, lm_d, c.Mcap)
    for _ in range(4):
        again = run_tree(sp, tb, lm_d, c.Mcap)
        for k in ("logits", "probs", "scores", "exit", "path_exit", "merged", "cols", "M"):
            assert np.array_equal(first[k], again[k], equal_nan=(first[k].dtype.kind == "f")), k
    for g_ in (0, G // 2, G - 1):      # and the same answers as a launch of that tree alone (different path)
        one = dict(ts[0], hidden=ts[g_]["hidden"], ids=ts[g_]["ids"], prev_probs=ts[g_]["prev_probs"],
                   parent=ts[g_]["parent"])   # the batch shares tree 0's norm weight and predictor
        single = run_tree(sp, one, lm_d, c.Mcap)
        close(first["scores"][g_], single["scores"], 1e-3, "sliced batch vs single tree")
        close(first["logits"][g_], single["logits"], 1.0, "sliced batch vs single tree logits")


def test_tree_throughput_configuration_sampled_trees(sp, oracle):
    """The 256-tree launch the benchmark times: integer outputs of every tree against numpy, all outputs of
    a sample of trees against the oracle."""
    c = synth.CONFIGS["C3"]
    lm_h, lm_d = lm_for(c)
    G = 256
    ts = [synth.make("C3", seed=1000 + i, lm=lm_h) for i in range(G)]
    tb = stack_trees(ts)
    got = run_tree(sp, tb, lm_d, c.Mcap)
    for g_ in range(G):
        u, inv = np.unique(ts[g_]["ids"], return_inverse=True)
        assert got["M"][g_] == len(u)
        assert np.array_equal(got["merged"][g_, :len(u)], u) and np.all(got["merged"][g_, len(u):] == -1)
        assert np.array_equal(got["cols"][g_].ravel(), inv.ravel())
    pick = [0, 17, 101, 255]
    sub = stack_trees([ts[i] for i in pick])
    sub = dict(sub, gamma=tb["gamma"], W1=tb["W1"], w2=tb["w2"], b1=tb["b1"], b2=tb["b2"])
    oracle.set_threads(8)
    ref = ref_tree(oracle, sub, c.Mcap)
    oracle.set_threads(1)
    check_tree({k: (v[pick] if v is not None else None) for k, v in got.items()}, ref, c.threshold, "256 x C3 sampled")


def test_tree_without_parent_and_with_malformed_parent(sp, oracle):
    t = synth.make("T4")
    c = t["cfg"]
    lm_d = dev(t["lm_head"])
    got = run_tree(sp, t, lm_d, c.Mcap, parent=None)
    assert got["path_exit"] is None
    ref = ref_tree(oracle, dict(t, parent=None), c.Mcap)
    check_tree(got, ref, c.threshold, "no parent")
    bad = t["parent"].copy()
    bad[5] = 9                                    # points forward: the path is refused, nothing loops
    got = run_tree(sp, t, lm_d, c.Mcap, parent=bad)
    assert got["path_exit"][5] == 0


def test_tree_merged_set_overflow_and_invalid_ids(sp, oracle):
    t = synth.make("T4")
    c = t["cfg"]
    lm_d = dev(t["lm_head"])
    true_M = len(np.unique(t["ids"]))
    got = run_tree(sp, t, lm_d, true_M - 1)
    assert got["M"] == true_M                     # the true size is reported
    assert np.all(np.isnan(got["scores"])) and got["exit"].sum() == 0 and got["path_exit"].sum() == 0
    t2 = dict(t, ids=t["ids"].copy())
    t2["ids"][4, 2] = c.V + 5
    t2["ids"][9, 0] = -1
    got = run_tree(sp, t2, lm_d, c.Mcap)
    u = np.unique(t2["ids"])
    assert got["M"] == len(u) and np.array_equal(got["merged"][:len(u)], u)
    good = np.ones(c.N, bool); good[[4, 9]] = False
    assert np.all(np.isnan(got["scores"][~good])) and np.all(got["exit"][~good] == 0)
    ref = ref_tree(oracle, t, c.Mcap)
    close(got["scores"][good], ref["scores"][good], 1e-3, "valid nodes beside invalid ones")


def test_tree_argument_errors(sp):
    t = synth.make("T4")
    c = t["cfg"]
    lm_d = dev(t["lm_head"])
    with pytest.raises(sp.SpeceeError) as ei:
        run_tree(sp, t, lm_d, c.Mcap, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == -3
    with pytest.raises(sp.SpeceeError) as ei:
        run_tree(sp, t, lm_d, 5000)
    assert ei.value.code == -1


def test_tree_is_deterministic(sp):
    t = synth.make("T3")
    lm_d = dev(t["lm_head"])
    a = run_tree(sp, t, lm_d, 96)
    b = run_tree(sp, t, lm_d, 96)
    for k in a:
        if a[k] is not None:
            assert np.array_equal(a[k], b[k]), k


def test_tree_c3_llama7b_60_nodes(sp, oracle):
    c = synth.CONFIGS["C3"]
    lm_h, lm_d = lm_for(c)
    for seed in range(3):
        t = synth.make("C3", seed=seed, lm=lm_h)
        oracle.set_threads(8)
        ref = ref_tree(oracle, t, c.Mcap)
        oracle.set_threads(1)
        got = run_tree(sp, t, lm_d, c.Mcap)
        e = check_tree(got, ref, c.threshold, f"C3 seed {seed}")
        print("C3 seed", seed, "M", int(ref["M"]), "exits", int(ref["exit"].sum()), "paths",
              int(ref["path_exit"].sum()), "worst", e)
        assert 0 < ref["exit"].sum() < c.N and ref["M"] <= 64


# ---------------------------------------------------------------- multi-state full head (matrix cores)
@pytest.mark.parametrize("d,V,N", [(64, 37, 3), (1032, 1001, 5), (4096, 515, 16), (520, 4100, 64), (2048, 300, 70)])
def test_lm_head_multi_state_small(sp, oracle, d, V, N):
    rng = np.random.default_rng(d + V + N)
    h = rng.standard_normal((N, d)).astype(np.float16)
    g = (1 + 0.05 * rng.standard_normal(d)).astype(np.float16)
    W = (0.05 * rng.standard_normal((V, d))).astype(np.float16)
    ref = oracle.lm_head_gemv(h, g, W)
    got = host(sp.lm_head_gemv(dev(h), dev(g), dev(W)))
    close(got, ref, 1.0, f"lm_head gemm d={d} V={V} N={N}")


def test_lm_head_16_states_llama13b_sampled_rows(sp, oracle):
    c = synth.CONFIGS["C4"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C4", lm=lm_h)
    h = t["hidden"][0]
    got = host(sp.lm_head_gemv(dev(h), dev(t["gamma"]), lm_d))
    rows = np.unique(np.concatenate([np.random.default_rng(0).integers(0, c.V, 2048), [0, c.V - 1],
                                     t["ids"].ravel()])).astype(np.int32)
    oracle.set_threads(8)
    ref = oracle.lm_head_rows(h, t["gamma"], lm_h, rows)
    oracle.set_threads(1)
    close(got[:, rows], ref, 1.0, "lm_head 32000x5120 N=16 sampled rows")


def test_c5_large_vocab_tree_and_full_head(sp, oracle):
    """d=8192, V=128256, K=8, 64-node tree; plus lm_head_gemv on the same hidden states (sampled rows)."""
    c = synth.CONFIGS["C5"]
    lm_h, lm_d = lm_for(c)
    t = synth.make("C5", lm=lm_h)
    oracle.set_threads(8)
    ref = ref_tree(oracle, t, c.Mcap)
    got = run_tree(sp, t, lm_d, c.Mcap)
    e = check_tree(got, ref, c.threshold, "C5")
    print("C5 M", int(ref["M"]), "exits", int(ref["exit"].sum()), "worst", e)
    assert ref["M"] <= 256 and 0 < ref["exit"].sum() < c.N
    full = host(sp.lm_head_gemv(dev(t["hidden"]), dev(t["gamma"]), lm_d))
    rows = np.unique(np.concatenate([np.random.default_rng(1).integers(0, c.V, 1024), [0, c.V - 1],
                                     ref["merged"][:int(ref["M"])]])).astype(np.int32)
    ref_rows = oracle.lm_head_rows(t["hidden"], t["gamma"], lm_h, rows)
    w = close(full[:, rows], ref_rows, 1.0, "lm_head 128256x8192 N=64 sampled rows")
    one = host(sp.lm_head_gemv(dev(t["hidden"][:1]), dev(t["gamma"]), lm_d))
    close(one[:, rows], ref_rows[:1], 1.0, "lm_head 128256x8192 N=1 sampled rows")
    oracle.set_threads(1)
    # the tree's logits are the full head's logits at the ids
    idx = t["ids"]
    close(got["logits"], np.take_along_axis(full, idx, axis=1), 1.0, "tree logits vs full head")
    print("C5 lm_head worst", w)
    # throughput mode at full size, as the benchmark launches it: 256 trees (one workgroup each) and 64 trees
    # (d-slices by ticket) of this shape per launch; sampled trees against the oracle, integer outputs of all
    oracle.set_threads(8)
    for G in (256, 64):
        ts = [synth.make("C5", seed=900 + i, lm=np.zeros((1, 1), np.float16)) for i in range(G)]
        for x in ts:
            for k in ("gamma", "W1", "w2", "b1", "b2"):
                x[k] = t[k]
        tb = stack_trees(ts)
        gotb = run_tree(sp, tb, lm_d, c.Mcap)
        assert np.all(np.isfinite(gotb["scores"]))
        for gi in (0, G // 2 + 1, G - 1):
            one = dict(ts[gi], lm_head=lm_h)
            r1 = ref_tree(oracle, one, c.Mcap)
            check_tree({k: v[gi] for k, v in gotb.items()}, r1, c.threshold, f"C5 batch of {G}, tree {gi}")
        for gi in range(G):  # merged sets of every tree: integer work, exact
            u = np.unique(ts[gi]["ids"])
            assert gotb["M"][gi] == len(u) and np.array_equal(gotb["merged"][gi][:len(u)], u)
    oracle.set_threads(1)
