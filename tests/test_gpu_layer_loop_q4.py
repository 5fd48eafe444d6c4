"""GPU: the early-exit decode loop in one persistent launch on the 4-bit group-quantised LM head
(specee_layer_loop_q4; paper Sec. 4.3.3 and 5.3 in the weight-quantised setting of Sec. 7.1 / 7.3) against the
oracle's loop on the same codes, scales and zero-points."""
import numpy as np
import pytest
import torch

from paper_2504_08850_amd import synth

from parity import close, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    specee.lib()
    return specee


def loop_inputs_q4(seed, d, V, K, H, L, B, group, bias=True):
    """Random model and tokens on a quantised head (the synthetic quantiser on a random fp16 head)."""
    rng = np.random.default_rng(seed)
    lm = (0.05 * rng.standard_normal((V, d))).astype(np.float16)
    q, scales, zeros = synth.quantize_q4(lm, group)
    return dict(
        hidden=rng.standard_normal((L, B, d)).astype(np.float16),
        gamma=(1 + 0.05 * rng.standard_normal(d)).astype(np.float16),
        q=q, scales=scales, zeros=zeros, group=group,
        ids=np.stack([rng.choice(V, K, replace=False) for _ in range(B)]).astype(np.int32),
        W1=(0.1 * rng.standard_normal((L, H, 3 * K))).astype(np.float16),
        w2=(0.1 * rng.standard_normal((L, H))).astype(np.float16),
        b1=(0.1 * rng.standard_normal((L, H))).astype(np.float16) if bias else None,
        b2=(0.1 * rng.standard_normal(L)).astype(np.float16) if bias else None)


def head(oracle, t, l, b):
    return oracle.lm_head_gemv_q4(t["hidden"][l][b:b + 1], t["gamma"], t["q"], t["scales"], t["zeros"], t["group"])[0]


def plant_hits(oracle, t, plant):
    """Token b's first id becomes the quantised head's arg-max at layer plant[b] (None: ids stay random)."""
    K = t["ids"].shape[1]
    for b, l in enumerate(plant):
        if l is None:
            continue
        tok = int(head(oracle, t, l, b).argmax())
        rest = [int(i) for i in t["ids"][b] if i != tok][:K - 1]
        t["ids"][b] = [tok] + rest
    return t


def reference(oracle, t, threshold, active=None):
    ref = oracle.layer_loop_q4(t["hidden"], t["gamma"], t["q"], t["scales"], t["zeros"], t["group"], t["ids"], t["W1"],
                               t["w2"], t["b1"], t["b2"], active=active, threshold=threshold)
    live = ref["scores"] != 0
    assert np.all(np.abs(ref["scores"][live] - threshold) > 1e-3), "pick another seed: a score sits on the threshold"
    # a verification's arg-max is only comparable when the runner-up is further away than the tolerance
    for l, b in zip(*np.nonzero(ref["exit"])):
        full = np.sort(head(oracle, t, l, b))
        assert full[-1] - full[-2] > 4e-3 * max(1.0, abs(full[-1])), "pick another seed: arg-max nearly tied"
    return ref


def check_loop(oracle, sp, t, threshold, active=None, what="", graph=False):
    ref = reference(oracle, t, threshold, active)
    args = [dev(t["hidden"]), dev(t["gamma"]), dev(t["q"].view(np.int32)), dev(t["scales"]), dev(t["zeros"]), t["group"],
            dev(t["ids"]), dev(t["W1"]), dev(t["w2"]), dev(t["b1"]), dev(t["b2"])]
    kw = dict(active=dev(active), threshold=threshold)
    out = sp.layer_loop_q4(*args, **kw)
    torch.cuda.synchronize()

    def compare(o, tag):
        g = {k: host(v) for k, v in o.items() if k != "_workspace"}
        assert np.all(g["status"] == 0), tag + " status"
        for k in ("exit", "ver_token", "hit", "exit_layer", "token"):
            assert np.array_equal(g[k], ref[k]), f"{what} {tag} {k}"
        close(g["logits"], ref["logits"], 1.0, f"{what} {tag} logits")
        close(g["probs"], ref["probs"], 1e-3, f"{what} {tag} probs")
        close(g["scores"], ref["scores"], 1e-3, f"{what} {tag} scores")
    compare(out, "eager")
    if graph:
        ws = out.pop("_workspace")
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            sp.layer_loop_q4(*args, out=out, workspace=ws, **kw)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            sp.layer_loop_q4(*args, out=out, workspace=ws, **kw)
        for rep in range(3):
            for k, x in out.items():
                if k != "_workspace":
                    x.fill_(7)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            compare(out, f"graph replay {rep}")
    return ref


CASES = [
    # seed, d, V, K, H, L, B, group, plant, threshold, bias
    (2, 1024, 301, 4, 512, 6, 7, 128, [0, 3, None, 5, 1, 2, 4], 0.45, True),   # 16-byte chunks, exits at every depth
    (2, 2048, 997, 8, 512, 5, 3, 64, [4, None, 2], 0.45, False),                # K = 8
    (2, 520, 777, 3, 100, 7, 5, 8, [6, 1, None, 3, 3], 0.48, True),             # word path (group 8), K odd, ragged d
    (3, 8192, 2000, 4, 1024, 4, 2, 256, [3, 1], 0.45, True),                    # two vectors per thread, H > 512
    (38, 1024, 1000, 4, 512, 6, 64, 32, [i % 6 if i % 5 else None for i in range(64)], 0.6, False),  # 64 tokens
]


@pytest.mark.parametrize("seed,d,V,K,H,L,B,group,plant,threshold,bias", CASES)
def test_layer_loop_q4_matches_oracle(sp, oracle, seed, d, V, K, H, L, B, group, plant, threshold, bias):
    t = plant_hits(oracle, loop_inputs_q4(seed, d, V, K, H, L, B, group, bias), plant)
    oracle.set_threads(8)
    ref = check_loop(oracle, sp, t, threshold, what=f"q4 loop d={d} K={K} B={B} group={group}", graph=(d == 1024 and B == 7))
    oracle.set_threads(1)
    assert ref["hit"].sum() >= 1 and (ref["exit"].sum() > ref["hit"].sum() or B <= 3)
    assert (ref["exit_layer"] >= 0).any()


def test_layer_loop_q4_active_mask_never_and_always_firing(sp, oracle):
    seed, d, V, K, H, L, B, group, plant, thr, bias = CASES[0]
    t = plant_hits(oracle, loop_inputs_q4(seed, d, V, K, H, L, B, group, bias), plant)
    active = np.array([0, 1, 1, 0, 1, 1], np.int32)
    ref = check_loop(oracle, sp, t, thr, active=active, what="q4 active mask")
    assert not ref["scores"][0].any() and not ref["scores"][3].any()
    ref = check_loop(oracle, sp, t, 2.0, what="q4 never fires")
    assert np.all(ref["exit_layer"] == -1) and not ref["exit"].any()
    ref = check_loop(oracle, sp, t, -1.0, what="q4 always fires")
    assert ref["exit"].sum() >= 15


def test_layer_loop_q4_llama7b_head(sp, oracle):
    """32 layers of one token at d=4096, V=32000, K=4, group 128, with an accepted verification on the way."""
    c = synth.CONFIGS["C2"]
    t0 = synth.make("C2", seed=4, bias=False)
    q, scales, zeros = synth.quantize_q4(t0["lm_head"], 128)
    t = dict(hidden=t0["hidden"], gamma=t0["gamma"], q=q, scales=scales, zeros=zeros, group=128, ids=t0["ids"].copy(),
             W1=t0["W1"], w2=t0["w2"], b1=None, b2=None)
    oracle.set_threads(8)
    t = plant_hits(oracle, t, [21])
    ref = check_loop(oracle, sp, t, 0.5, what="q4 7B shape")
    oracle.set_threads(1)
    assert ref["exit_layer"][0] >= 0 and ref["exit"].sum() >= 2
    print("q4 7B loop: fired at", np.flatnonzero(ref["exit"][:, 0]).tolist(), "exit", ref["exit_layer"].tolist())


def test_layer_loop_q4_empty_stack_and_argument_errors(sp):
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
    f16, i32 = torch.float16, torch.int32
    d, V, K, H, group = 64, 10, 4, 8, 32
    # an empty stack touches no input and reports "ran the whole stack"
    out = sp.layer_loop_q4(z((0, 3, d), f16), z((d,), f16), z((V, d // 8), i32), z((V, d // group), f16),
                           z((V, d // group), f16), group, z((3, K), i32), z((0, H, 3 * K), f16), z((0, H), f16))
    torch.cuda.synchronize()
    assert host(out["exit_layer"]).tolist() == [-1, -1, -1] and host(out["token"]).tolist() == [-1, -1, -1]
    assert host(out["status"]).tolist() == [0, 0, 0]
    L = 2
    base = lambda K_, group_: (z((L, 2, d), f16), z((d,), f16), z((V, d // 8), i32), z((V, d // group_), f16),
                                z((V, d // group_), f16), group_, z((2, K_), i32), z((L, H, 3 * K_), f16), z((L, H), f16))
    with pytest.raises(sp.SpeceeError) as ei:     # K beyond what the quantised loop keeps in registers
        sp.layer_loop_q4(*base(16, 32))
    assert ei.value.code == -1
    with pytest.raises(sp.SpeceeError) as ei:     # workspace too small
        sp.layer_loop_q4(*base(4, 32), workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == -3
