"""GPU check of specee_predict_tree_static, the tree entry point that allocates nothing: its outputs must
equal those of specee_predict_tree (same kernels, scratch in the library's static device array instead of
a caller's workspace) on two calls in a row, the second on a smaller input, so that whatever the first
call left in the shared array is seen not to matter.  Runs last: a failure here must not hide other tests."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2504_08850_amd import synth

from parity import dev, host

pytestmark = pytest.mark.gpu

KEYS = ("merged", "M", "cols", "logits", "probs", "scores", "exit", "path_exit")


@pytest.fixture(scope="module")
def sp():
    from paper_2504_08850_amd import specee
    specee.lib()
    assert torch.cuda.is_available()
    return specee


def stack(ts):
    st = lambda k: np.stack([t[k] for t in ts])
    return dict(ts[0], hidden=st("hidden"), ids=st("ids"), prev_probs=st("prev_probs"), parent=st("parent"))


def outputs(G, N, K, Mcap, fill):
    i32, f32 = torch.int32, torch.float32
    mk = lambda shape, dt: torch.full(shape, fill, dtype=dt, device="cuda")
    return dict(merged=mk((G, Mcap), i32), M=mk((G,), i32), cols=mk((G, N, K), i32), logits=mk((G, N, K), f32),
                probs=mk((G, N, K), f32), scores=mk((G, N), f32), exit=mk((G, N), i32), path_exit=mk((G, N), i32))


def both(sp, tb, Mcap):
    """(workspace entry point, static-scratch entry point) outputs for a batch of trees."""
    G, N, K = tb["ids"].shape
    a = [dev(tb[k]) for k in ("hidden", "gamma", "lm_head", "ids", "prev_probs", "W1", "w2", "b1", "b2")]
    par = dev(tb["parent"])
    ref = sp.predict_tree(*a, parent=par, Mcap=Mcap)
    out = outputs(G, N, K, Mcap, 7)          # pre-filled, so that an output left unwritten shows
    got = sp.predict_tree_static(*a, parent=par, Mcap=Mcap, out=out)
    torch.cuda.synchronize()
    return {k: host(ref[k]) for k in KEYS}, {k: host(got[k]) for k in KEYS}


def same(ref, got, what):
    for k in KEYS:
        assert np.array_equal(ref[k], got[k], equal_nan=(ref[k].dtype.kind == "f")), (what, k)


def test_static_scratch_entry_point_two_calls_in_a_row(sp, oracle):
    # first call: 24 trees -> eight d-slice workgroups per tree, accumulators and tickets in the scratch array
    ts = [synth.make("T3", seed=s) for s in range(24)]
    c = ts[0]["cfg"]
    big = stack(ts)
    ref, got = both(sp, big, c.Mcap)
    same(ref, got, "24 trees, ticketed d-slices")
    # against the oracle too (the bar of every parity test), on the static entry point's outputs
    orc = oracle.predict_tree(big["hidden"], big["gamma"], big["lm_head"], big["ids"], big["prev_probs"], big["W1"],
                              big["w2"], big["b1"], big["b2"], parent=big["parent"], Mcap=c.Mcap)
    assert np.array_equal(got["merged"], orc["merged"]) and np.array_equal(got["cols"], orc["cols"])
    err = np.abs(got["scores"] - orc["scores"]) / np.maximum(np.abs(orc["scores"]), 1e-3)
    assert err.max() <= 2e-3
    decided = np.abs(orc["scores"] - c.threshold) > 1e-4
    assert np.array_equal(got["exit"][decided], orc["exit"][decided])
    # second call, smaller: one tree -> d-split partial sums through the same array (other layout, other sizes)
    small = stack([synth.make("T4", seed=5)])
    ref, got = both(sp, small, small["cfg"].Mcap)
    same(ref, got, "one tree, d-split partial sums")
    # and the first input once more: tickets left behind by the earlier calls must have been cleared
    ref, got = both(sp, big, c.Mcap)
    same(ref, got, "24 trees again")


def test_static_scratch_limit_is_an_error_not_an_overrun(sp):
    """A call whose launch shape needs more than the static array holds is refused on the host."""
    d, V, K, H, N, Mcap, G = 8192, 64, 8, 64, 500, 4096, 4
    f16, i32, f32 = torch.float16, torch.int32, torch.float32
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
    with pytest.raises(sp.SpeceeError) as ei:
        sp.predict_tree_static(z((G, N, d), f16), z((d,), f16), z((V, d), f16), z((G, N, K), i32), z((G, N, K), f32),
                               z((H, 3 * K), f16), z((H,), f16), parent=z((G, N), i32), Mcap=Mcap,
                               out=outputs(G, N, K, Mcap, 0))
    assert ei.value.code == -5
    assert sp.lib().specee_strerror(C.c_int(-5)) not in (b"success", b"unknown status")
