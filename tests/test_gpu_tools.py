"""The measurement tools built on the verify step, run end to end on the GPU at small sizes."""
import json
import pytest

pytestmark = pytest.mark.gpu


def test_latency_model_fit_on_a_two_layer_model():
    """Forward-latency model of Sec. 4.2.1 (Eq. 1): verify-step time is linear in the number of processed tokens,
    t_fwd = c_base + c_tok * n_toks.  Measured on the 7B-width model cut to two layers over the long-tail contexts of
    config 3: positive slope and intercept, a good fit, and the report has the shape the tool documents."""
    from paper_2511_13841_amd.latency_model import sweep
    r = sweep("c3", ks=(0, 2, 4, 8, 16), steps=4, warmup=2, layers=2)
    json.dumps(r)                                   # JSON-able
    assert r["n_layers"] == 2 and r["batch"] == 128 and [row["k"] for row in r["sweep"]] == [0, 2, 4, 8, 16]
    assert [row["n_toks"] for row in r["sweep"]] == [128 * (k + 1) for k in (0, 2, 4, 8, 16)]
    fit = r["fit"]
    print("latency fit:", fit)
    assert fit["c_tok_ms"] > 0 and fit["c_base_ms"] > 0 and fit["r2"] > 0.9
    assert fit["mean_relative_error"] < 0.25        # the paper reports about 12 % for its own fit
    assert r["best_k"] in (0, 2, 4, 8, 16) and isinstance(r["over_proposing_hurts"], bool)


def test_projection_timing_with_and_without_arithmetic():
    """das_debug_gemm_time in both modes on the projections of config 4 (272 rows): the copies-only launch moves the same
    tiles behind the same barriers, so it cannot take much longer than the full launch, and for the few-row shapes --
    which Sec. 4.2.1 prices as c_base, the cost of moving parameters -- it is most of the time."""
    from paper_2511_13841_amd.gemm_shapes import measure
    r = measure("c4", iters=12)
    json.dumps(r)
    assert r["rows"] == 272 and [p["projection"] for p in r["projections"]] == ["qkv", "o", "gate_up", "down", "lm_head"]
    for p in r["projections"]:
        print(p)
        assert 1.0 < p["us"] < 5000.0 and 0.3 * p["us"] < p["us_copies_only"] < 1.15 * p["us"], p
        assert 0.0 < p["frac_of_floor"] <= 1.0, p
