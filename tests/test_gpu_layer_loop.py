"""GPU: the layer loop with device-side control -- predict, verification gated by the predictor's exit flag,
and a per-token done flag that switches off everything after the exit (paper Sec. 4.3.3 and Fig. 6: a token
leaves the model at the first layer whose predictor fires AND whose verification hits).  The host looks at no
flag between the launches; the expected values are composed from the oracle's predict and verify."""
import numpy as np
import pytest
import torch

from paper_2504_08850_amd import synth

from parity import close, dev, host

pytestmark = pytest.mark.gpu

THRESHOLD = 0.35


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    specee.lib()
    return specee


def make_case(oracle):
    t = synth.make("T2", seed=4, bias=True)
    c = t["cfg"]
    ids = t["ids"].copy()
    # let the verification hit at different layers: token b's first id is the full head's arg-max at layer b % L
    for b in range(c.B):
        full = oracle.lm_head_gemv(t["hidden"][b % c.L][b:b + 1], t["gamma"], t["lm_head"], eps=c.eps)[0]
        if b != 3:                                   # token 3 keeps random ids: it never hits
            ids[b, 0] = int(full.argmax())
            for k in range(1, c.K):                  # keep the ids distinct
                if ids[b, k] == ids[b, 0]:
                    ids[b, k] = (ids[b, 0] + 1 + k) % c.V
    return t, c, ids


def expected(oracle, t, c, ids):
    B, K, L = c.B, c.K, c.L
    done = np.zeros(B, bool)
    prev = np.zeros((B, K))
    out = []
    for l in range(L):
        e = dict(logits=np.zeros((B, K)), probs=prev.copy(), scores=np.zeros(B), exit=np.zeros(B, np.int32),
                 token=np.full(B, -1, np.int32), hit=np.zeros(B, np.int32), done_before=done.copy())
        live = np.flatnonzero(~done)
        if len(live):
            r = oracle.predict(t["hidden"][l][live], t["gamma"], t["lm_head"], ids[live], prev[live].astype(np.float32),
                               t["W1"][l], t["w2"][l], t["b1"][l], t["b2"][l], eps=c.eps, threshold=THRESHOLD)
            assert np.all(np.abs(r["scores"] - THRESHOLD) > 1e-3), "pick another seed: a score sits on the threshold"
            for key in ("logits", "probs", "scores", "exit"):
                e[key][live] = r[key]
            fired = live[r["exit"] != 0]
            if len(fired):
                v = oracle.verify(t["hidden"][l][fired], t["gamma"], t["lm_head"], ids[fired], eps=c.eps)
                e["token"][fired] = v["token"]
                e["hit"][fired] = v["hit"]
                done[fired[v["hit"] != 0]] = True
        prev = e["probs"].copy()
        out.append(e)
    return out, done


def run_loop(sp, T, c, lm_d, ids_d, state):
    """All launches of the L-layer loop on the current stream; nothing is read back in between."""
    state["done"].zero_()
    prev = state["zero"]
    for l in range(c.L):
        o = state["pred"][l]
        sp.predict(T["hidden"][l], T["gamma"], lm_d, ids_d, prev, T["W1"][l], T["w2"][l], T["b1"][l], T["b2"][l],
                   eps=c.eps, threshold=THRESHOLD, out=o, done=state["done"])
        sp.verify(T["hidden"][l], T["gamma"], lm_d, ids_d, gate=o["exit"], done=state["done"], eps=c.eps,
                  out=state["ver"][l], workspace=state["ws"])
        prev = o["probs"]


def check(state, exp, done_ref, c, what):
    for l in range(c.L):
        e, p, v = exp[l], state["pred"][l], state["ver"][l]
        close(host(p["logits"]), e["logits"], 1.0, f"{what} layer {l} logits")
        close(host(p["probs"]), e["probs"], 1e-3, f"{what} layer {l} probs")
        close(host(p["scores"]), e["scores"], 1e-3, f"{what} layer {l} scores")
        assert np.array_equal(host(p["exit"]), e["exit"]), f"{what} layer {l} exit flags"
        assert np.array_equal(host(v["hit"]), e["hit"]), f"{what} layer {l} hits"
        fired = e["exit"] != 0
        assert np.array_equal(host(v["token"])[fired], e["token"][fired]), f"{what} layer {l} tokens"
        assert np.all(host(v["token"])[~fired] == -1)
    assert np.array_equal(host(state["done"]) != 0, done_ref), what + " done flags"


def test_layer_loop_device_side_control(sp, oracle):
    t, c, ids = make_case(oracle)
    exp, done_ref = expected(oracle, t, c, ids)
    exits = sum(int(e["exit"].sum()) for e in exp)
    hits = sum(int(e["hit"].sum()) for e in exp)
    skipped = sum(int(e["done_before"].sum()) for e in exp)
    assert hits >= 2 and exits > hits and skipped >= 2 and not done_ref.all(), (exits, hits, skipped)

    T = {k: dev(v) for k, v in t.items() if k not in ("cfg", "lm_head", "ids")}
    lm_d, ids_d = dev(t["lm_head"]), dev(ids)
    B, K = c.B, c.K
    mk = lambda *shape, dt=torch.float32: torch.full(shape, 7, dtype=dt, device="cuda")   # poisoned outputs
    state = dict(done=torch.zeros(B, dtype=torch.int32, device="cuda"), zero=torch.zeros((B, K), device="cuda"),
                 pred=[dict(logits=mk(B, K), probs=mk(B, K), scores=mk(B), exit=mk(B, dt=torch.int32))
                       for _ in range(c.L)],
                 ver=[dict(token=mk(B, dt=torch.int32), max_logit=mk(B), hit=mk(B, dt=torch.int32))
                      for _ in range(c.L)],
                 ws=torch.empty(sp.workspace_bytes(sp.OP_VERIFY, sp.Dims(c.d, c.V, K, c.H, c.eps, THRESHOLD), B),
                                dtype=torch.uint8, device="cuda"))
    run_loop(sp, T, c, lm_d, ids_d, state)
    torch.cuda.synchronize()
    check(state, exp, done_ref, c, "eager")

    # the same loop as one HIP graph, replayed with the program's own work in between
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        run_loop(sp, T, c, lm_d, ids_d, state)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        run_loop(sp, T, c, lm_d, ids_d, state)
    for rep in range(3):
        for o in state["pred"] + state["ver"]:
            for x in o.values():
                x.fill_(7)
        state["done"].fill_(1)                       # the graph's own first node clears it
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(state, exp, done_ref, c, f"graph replay {rep}")


# ------------------------------------------------------------------ the same loop as ONE launch (specee_layer_loop)
def loop_inputs(seed, d, V, K, H, L, B, plant, bias=True):
    """Random model and tokens; token b's first id is the full head's arg-max at layer plant[b] (None: never)."""
    rng = np.random.default_rng(seed)
    t = dict(
        hidden=rng.standard_normal((L, B, d)).astype(np.float16),
        gamma=(1 + 0.05 * rng.standard_normal(d)).astype(np.float16),
        lm_head=(0.05 * rng.standard_normal((V, d))).astype(np.float16),
        ids=np.stack([rng.choice(V, K, replace=False) for _ in range(B)]).astype(np.int32),
        W1=(0.1 * rng.standard_normal((L, H, 3 * K))).astype(np.float16),
        w2=(0.1 * rng.standard_normal((L, H))).astype(np.float16),
        b1=(0.1 * rng.standard_normal((L, H))).astype(np.float16) if bias else None,
        b2=(0.1 * rng.standard_normal(L)).astype(np.float16) if bias else None)
    return t, plant


def plant_hits(oracle, t, plant):
    V = t["lm_head"].shape[0]
    K = t["ids"].shape[1]
    for b, l in enumerate(plant):
        if l is None:
            continue
        full = oracle.lm_head_gemv(t["hidden"][l][b:b + 1], t["gamma"], t["lm_head"])[0]
        tok = int(full.argmax())
        rest = [int(i) for i in t["ids"][b] if i != tok][:K - 1]
        t["ids"][b] = [tok] + rest
    return t


def check_loop(oracle, sp, t, threshold, active=None, what="", graph=False):
    L, B, d = t["hidden"].shape
    ref = oracle.layer_loop(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"],
                            active=active, threshold=threshold)
    live = ref["scores"] != 0
    assert np.all(np.abs(ref["scores"][live] - threshold) > 1e-3), "pick another seed: a score sits on the threshold"
    # a verification's arg-max is only comparable when the runner-up is further away than the tolerance
    for l, b in zip(*np.nonzero(ref["exit"])):
        full = np.sort(oracle.lm_head_gemv(t["hidden"][l][b:b + 1], t["gamma"], t["lm_head"])[0])
        assert full[-1] - full[-2] > 4e-3 * max(1.0, abs(full[-1])), "pick another seed: arg-max nearly tied"
    args = [dev(t[k]) for k in ("hidden", "gamma", "lm_head", "ids", "W1", "w2", "b1", "b2")]
    kw = dict(active=dev(active), threshold=threshold)
    out = sp.layer_loop(*args, **kw)
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
            sp.layer_loop(*args, out=out, workspace=ws, **kw)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            sp.layer_loop(*args, out=out, workspace=ws, **kw)
        for rep in range(3):
            for k, x in out.items():
                if k != "_workspace":
                    x.fill_(7)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            compare(out, f"graph replay {rep}")
    return ref


@pytest.mark.parametrize("seed,d,V,K,H,L,B,plant,threshold,bias", [
    (6, 1032, 301, 4, 512, 6, 7, [0, 3, None, 5, 1, 2, 4], 0.45, True),     # ragged d, planted exits at every depth
    (1, 2056, 997, 8, 512, 5, 3, [4, None, 2], 0.45, False),                # K = 8
    (1, 520, 777, 3, 100, 7, 5, [6, 1, None, 3, 3], 0.48, True),            # K odd: generic MLP path
    (1, 8192, 2000, 4, 1024, 4, 2, [3, 1], 0.45, True),                     # two vectors per thread, H > 512
    (4, 64, 40, 16, 8, 5, 4, [2, 2, None, 0], 0.5, True),                   # K = KMAX, tiny d
    (14, 1024, 1000, 4, 512, 6, 64, [i % 6 if i % 5 else None for i in range(64)], 0.6, False),  # 64 tokens: groups of 4
])
def test_layer_loop_one_launch_matches_oracle(sp, oracle, seed, d, V, K, H, L, B, plant, threshold, bias):
    t, plant = loop_inputs(seed, d, V, K, H, L, B, plant, bias)
    t = plant_hits(oracle, t, plant)
    oracle.set_threads(8)
    ref = check_loop(oracle, sp, t, threshold, what=f"loop d={d} K={K} B={B}", graph=(d == 1032))
    oracle.set_threads(1)
    assert ref["hit"].sum() >= 1 and (ref["exit"].sum() > ref["hit"].sum() or B <= 3)
    assert (ref["exit_layer"] >= 0).any() and (ref["exit_layer"] < L - 1).any()


def test_layer_loop_one_launch_active_mask_and_never_or_always_firing(sp, oracle):
    t, plant = loop_inputs(12, 1032, 301, 4, 512, 6, 7, [0, 3, None, 5, 1, 2, 4])
    t = plant_hits(oracle, t, plant)
    active = np.array([0, 1, 1, 0, 1, 1], np.int32)
    ref = check_loop(oracle, sp, t, 0.45, active=active, what="active mask")
    assert not ref["scores"][0].any() and not ref["scores"][3].any()
    ref = check_loop(oracle, sp, t, 2.0, what="never fires")              # no verification at all
    assert np.all(ref["exit_layer"] == -1) and not ref["exit"].any()
    ref = check_loop(oracle, sp, t, -1.0, what="always fires")            # a verification at every layer until the hit
    assert ref["exit"].sum() >= 20


def test_layer_loop_one_launch_llama7b_shape(sp, oracle):
    """The 32-layer sweep of one token at d=4096, V=32000, K=4 with an accepted verification on the way."""
    c = synth.CONFIGS["C2"]
    t = synth.make("C2", seed=4, bias=False)
    t = dict(t, ids=t["ids"].copy(), b1=None, b2=None)
    oracle.set_threads(8)
    # the drifting hidden state keeps its arg-max token over many layers, so the planted token is accepted at the
    # first layer from which it leads and whose predictor fires (layer 14 here, after four rejected verifications)
    t = plant_hits(oracle, t, [21])
    ref = check_loop(oracle, sp, t, 0.5, what="7B shape", graph=True)
    oracle.set_threads(1)
    assert ref["exit_layer"][0] == 14 and ref["exit"].sum() == 5
    print("7B loop: fired at", np.flatnonzero(ref["exit"][:, 0]).tolist(), "exit", ref["exit_layer"].tolist())


def test_layer_loop_bounded_wait_gives_up_instead_of_hanging(sp, oracle):
    """With a spin limit of one poll a group almost never meets: the call must still return, with status 1 for
    the tokens it gave up on (or 0 with correct results if the workgroups did arrive together)."""
    t, plant = loop_inputs(12, 1032, 3001, 4, 512, 4, 2, [1, 2])
    t = plant_hits(oracle, t, plant)
    args = [dev(t[k]) for k in ("hidden", "gamma", "lm_head", "ids", "W1", "w2", "b1", "b2")]
    out = sp.layer_loop(*args, threshold=-1.0, spin_limit=1)
    torch.cuda.synchronize()
    st = host(out["status"])
    assert set(st.tolist()) <= {0, 1}
    ref = oracle.layer_loop(t["hidden"], t["gamma"], t["lm_head"], t["ids"], t["W1"], t["w2"], t["b1"], t["b2"],
                            threshold=-1.0)
    ok = st == 0
    assert np.array_equal(host(out["exit_layer"])[ok], ref["exit_layer"][ok])
    assert np.all(host(out["exit_layer"])[~ok] == -1) and np.all(host(out["token"])[~ok] == -1)
    # the next call on the same workspace starts clean
    out2 = sp.layer_loop(*args, threshold=-1.0, workspace=out["_workspace"])
    torch.cuda.synchronize()
    assert np.all(host(out2["status"]) == 0) and np.array_equal(host(out2["exit_layer"]), ref["exit_layer"])


def test_layer_loop_deep_stack_with_a_sparse_active_mask(sp, oracle):
    """More than 128 layers (the mask no longer fits the two scalar words) with most predictors switched off."""
    L = 150
    t, _ = loop_inputs(3, 64, 40, 4, 8, L, 3, [None, None, None])
    rng = np.random.default_rng(5)
    active = (rng.random(L) < 0.3).astype(np.int32)
    active[[0, 63, 64, 127, 128, 149]] = [1, 1, 0, 1, 1, 1]
    ref = check_loop(oracle, sp, t, 2.0, active=active, what="deep stack, never fires")
    assert np.all(ref["scores"][active == 0] == 0) and np.all(ref["scores"][active == 1] != 0)
    t2, _ = loop_inputs(3, 64, 40, 4, 8, 100, 3, [None, None, None])      # 65..128 layers: both mask words
    a2 = (rng.random(100) < 0.4).astype(np.int32)
    a2[[0, 63, 64, 99]] = [0, 1, 1, 1]
    check_loop(oracle, sp, t2, 2.0, active=a2, what="100 layers, never fires")


def test_layer_loop_empty_stack_touches_no_input(sp):
    """L = 0: every token "runs the whole stack" (exit layer -1, token -1, status 0); the inputs may be empty."""
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
    f16, i32 = torch.float16, torch.int32
    d, V, K, H, B = 64, 10, 4, 8, 5
    out = sp.layer_loop(z((0, B, d), f16), z((d,), f16), z((V, d), f16), z((B, K), i32), z((0, H, 3 * K), f16),
                        z((0, H), f16))
    torch.cuda.synchronize()
    assert host(out["exit_layer"]).tolist() == [-1] * B and host(out["token"]).tolist() == [-1] * B
    assert host(out["status"]).tolist() == [0] * B


def test_layer_loop_argument_errors(sp):
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
    f16, i32 = torch.float16, torch.int32
    L, B, d, V, K, H = 2, 65, 64, 10, 4, 8
    with pytest.raises(sp.SpeceeError) as ei:     # more tokens than groups
        sp.layer_loop(z((L, B, d), f16), z((d,), f16), z((V, d), f16), z((B, K), i32), z((L, H, 3 * K), f16),
                      z((L, H), f16), workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == -1
    with pytest.raises(sp.SpeceeError) as ei:     # workspace too small
        sp.layer_loop(z((L, 2, d), f16), z((d,), f16), z((V, d), f16), z((2, K), i32), z((L, H, 3 * K), f16),
                      z((L, H), f16), workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == -3
