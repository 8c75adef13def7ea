"""The benchmark's output contract: one JSON line with the agreed keys, and a refusal of more than one GPU."""
import contextlib
import io
import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _run(argv):
    out, err = io.StringIO(), io.StringIO()
    with contextlib.redirect_stdout(out), contextlib.redirect_stderr(err):
        rc = bench.main(argv)
    return rc, out.getvalue(), err.getvalue()


def test_more_than_one_gpu_is_refused_with_a_message():
    rc, out, err = _run(["--gpus", "2"])
    assert rc != 0 and out.strip() == ""
    assert "one GPU" in err


def _visible_pairs(w, starts, prompt):
    """Brute force: (query, key) pairs of one prompt with pos_k <= pos_q, keys = imported module tokens + own tokens."""
    last = max(prompt.module_ids, key=lambda m: starts[m] + w.sizes[m])
    q_pos = [starts[last] + w.sizes[last] + i for i in range(prompt.n_new)]
    k_pos = [starts[m] + i for m in prompt.module_ids for i in range(w.sizes[m])] + q_pos
    return sum(1 for pq in q_pos for pk in k_pos if pk <= pq)


def test_attn_flops_counts_the_visible_pairs_only():
    """bench.attn_flops (the numerator of every TFLOP/s figure) against a brute-force count of visible
    (query, key) pairs, 4 x head_dim FLOPs per pair and query head, on small schemas with gaps and unions."""
    import oracle
    from paper_2311_04934_amd import workloads as W
    cases = [W.custom("flops_a", "bf16", 8, 2, 128, [37, 50, 21], None, [W.Prompt([0, 2], 9), W.Prompt([1], 1)], max_pos=256),
             W.custom("flops_b", "bf16", 4, 4, 64, [30, 64, 90, 17], [-1, 0, 0, -1], [W.Prompt([3, 1], 12), W.Prompt([0, 2, 3], 5)],
                      max_pos=512),
             W.tiny_fp32()]
    for w in cases:
        starts, _ = oracle.layout(w.sizes, w.union_ids)
        n_mod = [sum(w.sizes[m] for m in p.module_ids) for p in w.prompts]
        n_new = [p.n_new for p in w.prompts]
        pairs = sum(_visible_pairs(w, starts, p) for p in w.prompts)
        assert bench.attn_flops(w, n_mod, n_new) == 4 * w.head_dim * w.n_q_heads * pairs, w.name


def test_full_prefill_flop_count_against_the_papers_cost_model():
    """Sec. 2.2: a prefill over n tokens costs about 6 n d^2 + 4 n^2 d (d = hidden size); the 4 n^2 d term is the
    attention over ALL n^2 pairs.  Under the causal rule n(n+1)/2 pairs are visible, so the benchmark's count for
    'every token is a query' must be that term times (n+1)/(2n).  The formula is read from tests/golden/."""
    from paper_2311_04934_amd import workloads as W
    formulas = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "flops_model.txt")):
        if line.strip() and not line.startswith("#"):
            name, expr = line.split()
            formulas[name] = expr.replace("^", "**")
    for n, hq, dh in ((1000, 32, 128), (2240, 32, 128), (77, 4, 64)):
        d = hq * dh
        attention_term = eval(formulas["prefill"], {"n": n, "d": d}) - 6 * n * d * d
        assert attention_term == 4 * n * n * d
        w = W.custom("flops_full", "bf16", hq, hq, dh, [1], None, [W.Prompt([0], n)], max_pos=4096)
        assert bench.attn_flops(w, [0], [n]) * 2 * n == attention_term * (n + 1)
        # one decoding step over n cached tokens: the 4 n d term = one query seeing n keys
        assert eval(formulas["decode"], {"n": n, "d": d}) - 6 * d * d == bench.attn_flops(w, [n], [1]) - 4 * d


@pytest.mark.gpu
def test_default_workload_prints_one_json_line_with_the_agreed_keys():
    rc, out, _ = _run(["--layers", "2", "--steps", "2", "--warmup", "1", "--no-full-prefill"])
    assert rc == 0
    lines = [ln for ln in out.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 2 and j["warmup"] == 1
    assert j["vs_baseline"] is None and j["data"] == "synthetic" and j["dtype"] == "bf16"
    assert j["higher_is_better"] is True and j["value"] > 0 and j["ms_per_step"] > 0
    assert j["config"]["workload"] == "long_doc_8k" and "model" not in j["config"]
    r = j["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    # measured HBM bytes per launch: present only when profiles/ holds a record made on these very sources
    assert r["traffic"] is None or r["traffic"] > 0
    assert r["with_split_merge"]["frac"] <= r["frac"] and j["roofline_assemble"]["bound"] == "hbm"
    c = j["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["sample"] and c["unit"]
