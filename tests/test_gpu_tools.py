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


def test_copy_ring_probe_shows_what_bounds_the_copy_streams():
    """das_debug_copy_ring, the kernels' HBM/L2 -> LDS ring by itself.  What the kernel design rests on: (i) with few
    busy CUs a stream of L2 misses does not speed up with a deeper ring (a cap on what one CU keeps in flight, not the
    ring, bounds it); (ii) the non-temporal hint raises that stream's rate; (iii) copies that hit L2 arrive at more
    than twice the rate of misses; (iv) with every CU busy a pure miss stream is bound by HBM, far below the sum of
    the per-CU rates."""
    import paper_2511_13841_amd as das
    rate = lambda wgs, st, cp, sh, nt=False: (lambda us, nb: nb / us / 1e3 / wgs)(*das.debug_copy_ring(wgs, st, cp, sh, tiles=256, non_temporal=nt))
    miss4, miss9 = rate(32, 4, 4, 0), rate(32, 9, 4, 0)
    miss_nt, hit = rate(32, 4, 4, 0, True), rate(32, 4, 4, 4)
    full = rate(256, 4, 4, 0, True)
    print(f"GB/s per CU: misses {miss4:.1f} (4 stages) {miss9:.1f} (9 stages), non-temporal {miss_nt:.1f}, hits {hit:.1f}; all CUs non-temporal {full:.1f} = {full * 256 / 1e3:.2f} TB/s")
    assert 20.0 < miss4 < 200.0
    assert miss9 < 1.2 * miss4                   # (i)
    assert miss_nt > 1.3 * miss4                 # (ii)
    assert hit > 2.0 * miss4                     # (iii)
    assert 4.0 < full * 256 / 1e3 < 8.0          # (iv) TB/s, under the 8 TB/s peak
    assert full < 0.6 * miss_nt
    with pytest.raises(das.DasError):
        das.debug_copy_ring(32, 7, 4, 0)         # unsupported ring shape


def test_mfma_loop_probe_gives_the_ceiling_the_gemm_fractions_are_read_against():
    """das_debug_mfma_loop, the matrix pipe by itself: a 32x32x16 bf16 MFMA occupies its SIMD for about 32 shader cycles in
    every mode, the rate of the chip stays under the published 2.5 PFLOP/s, and the loop that reads random operands from
    LDS runs at a lower shader clock -- and so a lower rate -- than the loop on constant registers (the chip holds its
    power by lowering the clock): the GEMM kernels cannot beat the last mode's rate."""
    import paper_2511_13841_amd as das
    res = {m: das.debug_mfma_loop(m, 3000) for m in (0, 1, 2)}
    for m, (ns, ghz, pf) in res.items():
        print(f"mfma loop mode {m}: {ns:.2f} ns per MFMA, {ns * ghz:.1f} cycles, {ghz:.2f} GHz, {pf:.3f} PFLOP/s")
        assert 0.8 < ghz < 2.6 and 28.0 < ns * ghz < 48.0 and 0.5 < pf < 2.5
    assert res[1][2] < res[0][2] * 1.10 and res[2][2] < res[0][2] * 1.10      # (margin for boxes whose power state differs)
    with pytest.raises(das.DasError):
        das.debug_mfma_loop(3)
