"""The deviation predictor around the GPU look-ahead (paper Sec. 3.2.2): logs from the kernels' routing,
forest on the host, its deviation fed back into ef_route_predict.  Checks that hold whatever the data:
a zero gain reproduces the plain look-ahead exactly, the deviation never changes the routing itself, and on
recurring prompts the refined look-ahead names at least as many of the experts really used."""
import sys

import pytest

from paper_2510_26730_amd import delta_bench, synth

pytestmark = pytest.mark.gpu


def test_deviation_refines_the_lookahead_on_recurring_prompts():
    print("delta forest: tiny config, 3 layers, 32 requests, 24 prompts", flush=True)
    sys.stdout.flush()
    cfg = synth.CONFIGS["tiny"]
    r = delta_bench.run(cfg, T=32, L=3, H=2, P=24, steps=1, warmup=1, log_steps=10, eval_steps=2, n_trees=4,
                        max_depth=10, gains=(0.0, 2.0))
    plain = r["lookahead_recall_plain"]
    assert r["lookahead_recall_with_delta"]["0.0"] == plain          # zero deviation = plain top-k of the logits
    refined = r["lookahead_recall_with_delta"]["2.0"]
    assert len(plain) == 2 and all(0.0 < p <= 1.0 for p in plain)
    assert sum(refined) >= sum(plain)
    assert r["examples"] == 10 * 32 * 3 * 2 and r["features"] == 16 + 2 + 3 * cfg.E
    assert set(r["bit_accuracy_by_step_size"]) == {"1", "2"}
    assert 0.5 < r["bit_accuracy_eval"] <= 1.0
    assert r["layer_loop_with_delta"]["delta_rows_found"] > 0.0
