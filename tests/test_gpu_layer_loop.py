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
