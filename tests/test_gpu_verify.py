"""GPU parity: specee_verify (arg-max of the full head + membership) against the oracle."""
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


def run_verify(sp, h, g, W_d, ids, gate=None):
    out = sp.verify(dev(h), dev(g), W_d, dev(ids), gate=None if gate is None else dev(gate))
    torch.cuda.synchronize()
    return {k: host(v) for k, v in out.items()}


def check_verify(got, full, ids, what):
    """full: oracle logits [N][V].  The arg-max is unique only if the runner-up is not within tolerance."""
    N = full.shape[0]
    top = np.argsort(-full, axis=1)[:, :2]
    for n in range(N):
        best, second = full[n, top[n, 0]], full[n, top[n, 1]] if full.shape[1] > 1 else -np.inf
        close([got["max_logit"][n]], [best], 1.0, what + " max logit")
        if best - second > 4e-3 * max(1.0, abs(best)):
            assert got["token"][n] == top[n, 0], f"{what}: token of state {n}"
            assert got["hit"][n] == int(top[n, 0] in ids[n]), f"{what}: hit of state {n}"
        else:
            assert got["token"][n] in top[n], what
        assert got["hit"][n] == int(got["token"][n] in ids[n])


@pytest.mark.parametrize("d,V,N,K", [(64, 37, 1, 3), (1032, 1001, 2, 4), (4096, 515, 5, 4), (520, 4100, 64, 8),
                                     (2048, 300, 70, 2), (8, 1, 1, 1), (16384, 100, 2, 4)])
def test_verify_small(sp, oracle, d, V, N, K):
    rng = np.random.default_rng(d + V + N)
    h = rng.standard_normal((N, d)).astype(np.float16)
    g = (1 + 0.05 * rng.standard_normal(d)).astype(np.float16)
    W = (0.05 * rng.standard_normal((V, d))).astype(np.float16)
    full = oracle.lm_head_gemv(h, g, W)
    ids = rng.integers(0, V, size=(N, K)).astype(np.int32)
    ids[::2, 0] = full.argmax(axis=1)[::2]          # half of the states hit
    got = run_verify(sp, h, g, dev(W), ids)
    check_verify(got, full, ids, f"verify d={d} V={V} N={N}")
    ref = oracle.verify(h, g, W, ids)
    assert got["hit"].sum() > 0 or N == 1
    assert np.array_equal(ref["token"], full.argmax(axis=1))


def test_verify_tie_goes_to_lowest_id(sp):
    rng = np.random.default_rng(5)
    for N in (1, 4):
        h = rng.standard_normal((N, 256)).astype(np.float16)
        g = np.ones(256, np.float16)
        W = (0.01 * rng.standard_normal((700, 256))).astype(np.float16)
        boost = (0.5 * np.sign(h[0].astype(np.float32))).astype(np.float16)
        W[611] = boost
        W[87] = boost                                # identical rows: identical logits for state 0
        ids = np.tile(np.array([[611, 3]], np.int32), (N, 1))
        got = run_verify(sp, h, g, dev(W), ids)
        assert got["token"][0] == 87 and got["hit"][0] == 0


def test_verify_llama7b_and_agreement_with_lm_head(sp, oracle):
    c = synth.CONFIGS["C1"]
    lm_h = synth.lm_head(c.V, c.d, synth.lm_seed(c))
    lm_d = dev(lm_h)
    t = synth.make("C1", seed=2, lm=lm_h)
    oracle.set_threads(8)
    full = oracle.lm_head_gemv(t["hidden"], t["gamma"], lm_h)
    oracle.set_threads(1)
    ids = t["ids"].copy()
    got = run_verify(sp, t["hidden"], t["gamma"], lm_d, ids)
    check_verify(got, full, ids, "verify 32000x4096 miss")
    ids[0, 3] = full.argmax()
    got = run_verify(sp, t["hidden"], t["gamma"], lm_d, ids)
    check_verify(got, full, ids, "verify 32000x4096 hit")
    assert got["hit"][0] == 1
    # 16 states through the matrix-core path agree with the stored-logits path
    hid = synth.hidden(16, c.d, 77)
    gpu_full = host(sp.lm_head_gemv(dev(hid), dev(t["gamma"]), lm_d))
    ids16 = np.tile(ids, (16, 1))
    got = run_verify(sp, hid, t["gamma"], lm_d, ids16)
    assert np.array_equal(got["token"], gpu_full.argmax(axis=1))
    np.testing.assert_array_equal(got["max_logit"], gpu_full.max(axis=1))


@pytest.mark.parametrize("d,V,N,K,pattern", [(256, 700, 1, 4, "none"), (256, 700, 1, 4, "all"),
                                             (1032, 1001, 2, 4, "alternate"), (520, 4100, 5, 4, "alternate"),
                                             (520, 4100, 70, 8, "blocks"), (520, 4100, 70, 8, "none"),
                                             (520, 4100, 40, 2, "random")])
def test_verify_gated(sp, oracle, d, V, N, K, pattern):
    """Verification follows a positive prediction only (Sec. 4.3.3): states whose gate is 0 are skipped on
    the device and report token -1, max_logit 0, hit 0; the others match the ungated result."""
    rng = np.random.default_rng(d + V + N + len(pattern))
    h = rng.standard_normal((N, d)).astype(np.float16)
    g = (1 + 0.05 * rng.standard_normal(d)).astype(np.float16)
    W = (0.05 * rng.standard_normal((V, d))).astype(np.float16)
    full = oracle.lm_head_gemv(h, g, W)
    ids = rng.integers(0, V, size=(N, K)).astype(np.int32)
    ids[:, 0] = full.argmax(axis=1)
    gate = {"none": np.zeros(N, np.int32), "all": np.ones(N, np.int32),
            "alternate": (np.arange(N) % 2).astype(np.int32),
            "blocks": ((np.arange(N) // 16) % 2 * 7).astype(np.int32),     # whole 16-state blocks off, any non-zero = on
            "random": rng.integers(0, 2, N).astype(np.int32)}[pattern]
    W_d = dev(W)
    # poison the outputs first so that skipped states are seen to be written
    out = {"token": torch.full((N,), 123, dtype=torch.int32, device="cuda"),
           "max_logit": torch.full((N,), 9.0, dtype=torch.float32, device="cuda"),
           "hit": torch.full((N,), 5, dtype=torch.int32, device="cuda")}
    sp.verify(dev(h), dev(g), W_d, dev(ids), gate=dev(gate), out=out)
    torch.cuda.synchronize()
    got = {k: host(v) for k, v in out.items()}
    on = gate != 0
    assert np.all(got["token"][~on] == -1) and np.all(got["hit"][~on] == 0) and np.all(got["max_logit"][~on] == 0)
    if on.any():
        sub = {k: v[on] for k, v in got.items()}
        check_verify(sub, full[on], ids[on], f"gated verify {pattern} N={N}")
        ungated = run_verify(sp, h, g, W_d, ids)
        for k in got:
            assert np.array_equal(got[k][on], ungated[k][on]), k


def test_predict_then_gated_verify(sp, oracle):
    """The predictor's exit flags feed the verification without leaving the device."""
    c = synth.CONFIGS["T1"]
    t = synth.make("T1", seed=11, bias=True)
    lm_h = t["lm_head"]
    for threshold in (0.3, 0.5, 0.7):      # different mixes of exits
        ref = oracle.predict(t["hidden"], t["gamma"], lm_h, t["ids"], t["prev_probs"], t["W1"], t["w2"], t["b1"],
                             t["b2"], eps=c.eps, threshold=threshold)
        lm_d, hid_d, g_d, ids_d = dev(lm_h), dev(t["hidden"]), dev(t["gamma"]), dev(t["ids"])
        res = sp.predict(hid_d, g_d, lm_d, ids_d, dev(t["prev_probs"]), dev(t["W1"]), dev(t["w2"]), dev(t["b1"]),
                         dev(t["b2"]), eps=c.eps, threshold=threshold)
        out = sp.verify(hid_d, g_d, lm_d, ids_d, gate=res["exit"], eps=c.eps)
        torch.cuda.synchronize()
        flags = host(res["exit"])
        sure = np.abs(ref["scores"] - threshold) > 1e-4
        assert np.array_equal(flags[sure], ref["exit"][sure])
        vref = oracle.verify(t["hidden"], t["gamma"], lm_h, t["ids"], eps=c.eps)
        full = oracle.lm_head_gemv(t["hidden"], t["gamma"], lm_h, eps=c.eps)
        tok, hit = host(out["token"]), host(out["hit"])
        for n in range(c.B):
            if flags[n]:
                assert hit[n] == int(tok[n] in t["ids"][n])
                if tok[n] != vref["token"][n]:      # only a near-tie may differ
                    assert abs(full[n, tok[n]] - full[n].max()) <= 4e-3 * max(1.0, abs(full[n].max()))
            else:
                assert tok[n] == -1 and hit[n] == 0
