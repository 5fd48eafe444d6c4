"""CPU checks of the host side: the benchmark's command-line contract, the separation between the product
path and the oracle, and the synthetic-input recipes (shapes and structure of the paper's workloads)."""
import pathlib
import re
import subprocess
import sys

import numpy as np

from paper_2504_08850_amd import synth

ROOT = pathlib.Path(__file__).resolve().parents[1]


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""  # no JSON line for a run that measured nothing


def test_product_path_does_not_touch_the_oracle():
    """Only tests, the smoke check and the benchmark's cpu_baseline leg may use oracle/."""
    pkg = ROOT / "paper_2504_08850_amd"
    files = [p for p in pkg.rglob("*") if p.suffix in (".py", ".hip", ".h", ".cpp")]
    assert len(files) > 10
    for p in files:
        text = p.read_text()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f"{p} imports the oracle"
        assert "specee_oracle" not in text and "specee_ref" not in text, f"{p} names an oracle module or symbol"
    # and the oracle uses nothing of the product
    for p in (ROOT / "oracle").glob("*"):
        if p.suffix in (".py", ".c", ".h"):
            text = p.read_text()
            assert "paper_2504_08850_amd" not in text and "libspecee.so" not in text, p


def test_no_cpu_fallback_in_the_binding():
    text = (ROOT / "paper_2504_08850_amd" / "specee.py").read_text()
    assert "FileNotFoundError" in text
    for word in ("torch.matmul", "torch.softmax", "F.softmax", "torch.nn", ".cpu()"):
        assert word not in text, f"the binding computes something: {word}"


def test_c3_tree_recipe():
    c = synth.CONFIGS["C3"]
    ms = []
    for seed in range(12):
        t = synth.make("C3", seed=seed, lm=np.zeros((1, 1), np.float16))
        ids, parent = t["ids"], t["parent"]
        assert ids.shape == (c.N, c.K) and parent.shape == (c.N,)
        assert ids.min() >= 0 and ids.max() < c.V
        assert all(len(set(row)) == c.K for row in ids.tolist())          # distinct ids per node
        assert np.all(parent < np.arange(c.N)) and np.all(parent >= -1)   # parents precede children
        assert (parent == -1).sum() == 4                                  # first level of the tree
        assert np.bincount(parent[parent >= 0], minlength=c.N).max() <= 4  # branching 1-4
        depth = np.zeros(c.N, int)
        for n in range(c.N):
            depth[n] = 0 if parent[n] < 0 else depth[parent[n]] + 1
        assert depth.max() == 5 and np.bincount(depth).tolist() == [4, 8, 12, 14, 12, 10]
        ms.append(len(np.unique(ids)))
    assert 40 <= min(ms) and max(ms) <= c.Mcap  # the union stays within the merged-set capacity


def test_c5_tree_recipe_and_c4_overlap():
    c5 = synth.CONFIGS["C5"]
    t = synth.make("C5", seed=1, lm=np.zeros((1, 1), np.float16))
    assert t["ids"].shape == (c5.N, c5.K) and t["hidden"].shape == (c5.N, c5.d)
    m = len(np.unique(t["ids"]))
    assert 100 <= m <= c5.Mcap
    c4 = synth.CONFIGS["C4"]
    t4 = synth.make("C4", seed=1, lm=np.zeros((1, 1), np.float16))
    assert t4["hidden"].shape == (c4.L, c4.B, c4.d)
    assert 16 <= len(np.unique(t4["ids"])) <= c4.B * c4.K  # Zipf ranks: sequences share rows


def test_generators_are_seeded_and_fp16():
    a = synth.hidden(3, 64, 7)
    b = synth.hidden(3, 64, 7)
    assert a.dtype == np.float16 and np.array_equal(a, b)
    assert not np.array_equal(a, synth.hidden(3, 64, 8))
    p = synth.prob_rows(5, 4, 3)
    assert p.dtype == np.float32 and np.allclose(p.sum(axis=1), 1, atol=1e-6) and np.all(p > 0)
    ids = synth.ids_uniform_distinct(9, 4, 100, 2)
    assert ids.dtype == np.int32 and all(len(set(r)) == 4 for r in ids.tolist())


def test_quantize_q4_round_trip_error_is_half_a_step():
    rng = np.random.default_rng(0)
    w = (0.02 * rng.standard_normal((40, 256))).astype(np.float16)
    q, scales, zeros = synth.quantize_q4(w, 64)
    assert q.dtype == np.uint32 and q.shape == (40, 32) and scales.shape == (40, 4) and zeros.shape == (40, 4)
    codes = np.stack([(q >> (4 * e)) & 0xF for e in range(8)], axis=-1).reshape(40, 256).astype(np.float64)
    s = np.repeat(scales.astype(np.float64), 64, axis=1)
    z = np.repeat(zeros.astype(np.float64), 64, axis=1)
    back = s * (codes - z)
    # min/max rounding: every element within about half a step of its group (fp16 scale and zero-point)
    assert np.all(np.abs(back - w.astype(np.float64)) <= 0.75 * s + 1e-6)


def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers():
    """The C oracle and the library's host-side scheduler, built with -fsanitize=address,undefined and driven
    over every entry point (tests/sanitize/sanitize_main.c): no report, exit status 0."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("sanitize_host", ROOT / "tests" / "sanitize" / "build_and_run.py")
    sanitize = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(sanitize)
    r = sanitize.run()
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
    assert "ok" in r.stdout
