"""Helpers shared by the GPU parity tests: upload seeded inputs, compare against the oracle.

Tolerances: max relative error 2e-3 (fp16 inputs, fp32 accumulation), measured as
|gpu - ref| <= 2e-3 * max(|ref|, floor) with floor 1.0 for logits (their standard
deviation is 1.3-1.8, cancellation near zero makes a pure ratio meaningless) and
1e-3 for probabilities and scores.  Exit flags must be bit-exact unless the oracle
score lies within 1e-4 of the threshold.
"""
import numpy as np
import torch

RTOL = 2e-3
BAND = 1e-4


def dev(a, device="cuda"):
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def host(t):
    return None if t is None else t.detach().cpu().numpy()


def close(got, ref, floor, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite GPU output"
    err = np.abs(got - ref) / np.maximum(np.abs(ref), floor)
    worst = float(err.max()) if err.size else 0.0
    assert worst <= RTOL, f"{what}: max relative error {worst:.3e} > {RTOL}"
    return worst


def check_scored(got, ref, threshold, what=""):
    """got: dict of numpy arrays from the GPU; ref: oracle dict.  Returns worst errors."""
    e = {}
    e["logits"] = close(got["logits"], ref["logits"], 1.0, what + " logits")
    e["probs"] = close(got["probs"], ref["probs"], 1e-3, what + " probs")
    e["scores"] = close(got["scores"], ref["scores"], 1e-3, what + " scores")
    np.testing.assert_allclose(got["probs"].sum(axis=-1), 1.0, atol=1e-5, err_msg=what + " softmax sum")
    decided = np.abs(ref["scores"] - threshold) > BAND
    assert np.array_equal(got["exit"][decided], ref["exit"][decided]), what + " exit flags"
    assert set(np.unique(got["exit"]).tolist()) <= {0, 1}
    return e
