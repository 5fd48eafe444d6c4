"""GPU parity: specee_predict_tree_q4 (merged tree mapping on the 4-bit group-quantised LM head) against the
oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2504_08850_amd import synth

from parity import close, dev, host
from test_gpu_q4 import words
from test_gpu_tree import check_tree

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    specee.lib()
    return specee


def make(seed, d, V, K, H, N, G, group, Mcap, bias=False, head=None):
    rng = np.random.default_rng(seed)
    if head is None:
        w = (0.05 * rng.standard_normal((V, d))).astype(np.float16)
        head = synth.quantize_q4(w, group)
    ids = np.empty((G, N, K), np.int32)
    for g in range(G):
        width = [Mcap, max(K, Mcap - 9), max(K, Mcap // 2), K][g % 4]
        pool = rng.permutation(V)[:width]
        ids[g] = pool[rng.integers(0, width, size=(N, K))]
    return dict(
        hidden=rng.standard_normal((G, N, d)).astype(np.float16),
        gamma=(1 + 0.05 * rng.standard_normal(d)).astype(np.float16),
        q=head[0], scales=head[1], zeros=head[2], group=group, ids=ids,
        prev_probs=rng.dirichlet(np.ones(K), size=(G, N)).astype(np.float32),
        parent=np.tile(np.array([-1] + [int(rng.integers(0, n)) for n in range(1, N)], np.int32), (G, 1)),
        W1=(0.1 * rng.standard_normal((H, 3 * K))).astype(np.float16),
        w2=(0.1 * rng.standard_normal(H)).astype(np.float16),
        b1=(0.1 * rng.standard_normal(H)).astype(np.float16) if bias else None,
        b2=(0.1 * rng.standard_normal(1)).astype(np.float16) if bias else None)


def run(sp, t, Mcap, qd=None, parent="auto", ids=None):
    qd = qd or (words(t["q"]), dev(t["scales"]), dev(t["zeros"]))
    par = t["parent"] if isinstance(parent, str) else parent
    out = sp.predict_tree_q4(dev(t["hidden"]), dev(t["gamma"]), *qd, t["group"], dev(t["ids"] if ids is None else ids),
                             dev(t["prev_probs"]), dev(t["W1"]), dev(t["w2"]), dev(t["b1"]), dev(t["b2"]),
                             parent=dev(par), Mcap=Mcap)
    torch.cuda.synchronize()
    res = {k: host(v) for k, v in out.items()}
    res["parent"] = par
    return res


def ref(oracle, t, Mcap, parent="auto"):
    par = t["parent"] if isinstance(parent, str) else parent
    return oracle.predict_tree_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], t["group"], t["ids"],
                                  t["prev_probs"], t["W1"], t["w2"], t["b1"], t["b2"], parent=par, Mcap=Mcap)


@pytest.mark.parametrize("d,V,K,H,N,G,group,Mcap,bias", [
    (256, 300, 4, 64, 20, 1, 32, 64, False),      # one small tree, smallest group (a fold at every k-step)
    (1024, 900, 4, 512, 60, 3, 128, 64, True),    # the 60-node shape
    (2048, 777, 8, 512, 30, 5, 64, 128, False),   # K = 8, eight row tiles
    (544, 500, 3, 100, 37, 2, 32, 96, True),      # d not a multiple of the stage, K odd
    (8192, 700, 5, 200, 64, 2, 256, 128, False),  # a group spans two stages; full 64 nodes
    (4096, 2000, 4, 512, 60, 9, 128, 64, False),  # the 7B tree shape on a small vocabulary
    (64, 40, 16, 8, 5, 2, 32, 40, True),          # K = KMAX, tiny
    (32, 9, 1, 1, 1, 1, 32, 1, False),            # smallest legal tree
    (10240, 64, 4, 64, 20, 2, 32, 64, True),      # so many groups that the scales leave room for the short stage only
    (1280, 300, 8, 128, 33, 3, 320, 64, False),   # group neither a power of two nor a divisor of the stage
])
def test_tree_q4_shapes(sp, oracle, d, V, K, H, N, G, group, Mcap, bias):
    t = make(d + N + K, d, V, K, H, N, G, group, min(Mcap, V), bias)
    oracle.set_threads(8)
    r = ref(oracle, t, Mcap)
    oracle.set_threads(1)
    check_tree(run(sp, t, Mcap), r, 0.5, f"tree_q4 d={d} K={K} N={N} G={G} group={group}", min_compared=0.3)


def test_tree_q4_equals_independent_quantised_predictors_on_gpu(sp):
    t = make(7, 1024, 900, 4, 512, 60, 2, 128, 64)
    qd = (words(t["q"]), dev(t["scales"]), dev(t["zeros"]))
    tree = run(sp, t, 64, qd=qd)
    for g in range(2):
        ind = sp.predict_q4(dev(t["hidden"][g]), dev(t["gamma"]), *qd, 128, dev(t["ids"][g]), dev(t["prev_probs"][g]),
                            dev(t["W1"]), dev(t["w2"]))
        torch.cuda.synchronize()
        close(tree["logits"][g], host(ind["logits"]), 1.0, "tree_q4 vs independent logits")
        close(tree["scores"][g], host(ind["scores"]), 1e-3, "tree_q4 vs independent scores")


def test_tree_q4_overflow_invalid_ids_and_no_parent(sp, oracle):
    t = make(9, 512, 400, 4, 64, 24, 6, 64, 64)
    Ms = [len(np.unique(x)) for x in t["ids"]]
    cap = sorted(Ms)[len(Ms) // 2]
    got = run(sp, t, cap)
    assert np.array_equal(got["M"], np.array(Ms))
    over = np.array(Ms) > cap
    assert over.any() and not over.all()
    assert np.all(np.isnan(got["scores"][over])) and got["exit"][over].sum() == 0 and got["path_exit"][over].sum() == 0
    r = ref(oracle, t, 64)
    close(got["scores"][~over], r["scores"][~over], 1e-3, "trees that fit beside trees that overflow")
    bad = t["ids"].copy()
    bad[3, 4, 1] = 400
    bad[5, 0, 0] = -3
    got = run(sp, t, 64, parent=None, ids=bad)
    assert got["path_exit"] is None
    assert np.isnan(got["scores"][3, 4]) and np.isnan(got["scores"][5, 0]) and got["exit"][3, 4] == 0
    mask = np.ones((6, 24), bool); mask[3, 4] = mask[5, 0] = False
    close(got["scores"][mask], r["scores"][mask], 1e-3, "valid nodes beside invalid ones")
    u = np.unique(bad[5])
    assert got["M"][5] == len(u) and np.array_equal(got["merged"][5][:len(u)], u)


def test_tree_q4_llama7b_head_batch_of_trees(sp, oracle):
    """24 trees of the 60-node shape against the 32000 x 4096 head quantised in groups of 128."""
    c = synth.CONFIGS["C3"]
    lm_h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
    head = synth.quantize_q4(lm_h, 128)
    ts = [synth.make("C3", seed=200 + s, lm=lm_h) for s in range(24)]
    st = lambda k: np.stack([x[k] for x in ts])
    t = dict(hidden=st("hidden"), gamma=ts[0]["gamma"], q=head[0], scales=head[1], zeros=head[2], group=128,
             ids=st("ids"), prev_probs=st("prev_probs"), parent=st("parent"), W1=ts[0]["W1"], w2=ts[0]["w2"],
             b1=None, b2=None)
    oracle.set_threads(8)
    r = ref(oracle, t, c.Mcap)
    oracle.set_threads(1)
    got = run(sp, t, c.Mcap)
    e = check_tree(got, r, c.threshold, "24 x 60-node trees on the quantised 7B head")
    print("tree_q4 7B worst", e)
    assert 0 < r["exit"].sum() < r["exit"].size


def test_tree_q4_argument_errors(sp):
    t = make(1, 256, 100, 4, 64, 20, 1, 32, 64)
    with pytest.raises(sp.SpeceeError) as ei:       # Mcap beyond the eight row tiles
        run(sp, t, 200)
    assert ei.value.code == -1
    t16 = make(2, 256, 100, 4, 64, 20, 1, 16, 64)   # group must be a multiple of 32 here
    with pytest.raises(sp.SpeceeError) as ei:
        run(sp, t16, 64)
    assert ei.value.code == -1
    big = make(3, 64, 100, 4, 8, 65, 1, 32, 64)     # more than 64 nodes
    with pytest.raises(sp.SpeceeError) as ei:
        run(sp, big, 64)
    assert ei.value.code == -1
