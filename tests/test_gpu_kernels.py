"""GPU checks of single kernels through the C ABI (MFMA GEMM, KV page layout)."""
import numpy as np
import pytest

import das_inputs as di

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def das():
    import paper_2511_13841_amd as d
    return d


@pytest.mark.parametrize("M,N,K", [(20, 512, 256), (272, 384, 704), (130, 2048, 256), (1, 32, 64), (300, 1408, 256), (520, 16512, 192), (257, 16384, 64), (560, 16640, 192),
                                   (40, 320, 1024), (300, 256, 3584), (530, 192, 3136), (64, 128, 16448), (513, 96, 16384),
                                   (600, 16384, 64), (1030, 16448, 320), (320, 16400, 128), (450, 16384, 192),
                                   (272, 2048, 16384), (160, 2176, 16448), (230, 2048, 16384),
                                   (700, 400, 16384), (1090, 200, 18944), (2250, 2048, 16384)])      # many rows, long K: the two halves of K in two workgroups; or grouped in one
def test_mfma_gemm_against_fp64(das, M, N, K):
    rng = np.random.default_rng(M * 7 + N)
    a = di.f32_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    w = di.f32_to_bf16(rng.standard_normal((N, K)).astype(np.float32) * 0.05)
    print(f"gemm M={M} N={N} K={K}", flush=True)
    c = das.debug_gemm(a, w)
    ref = di.bf16_to_f32(a).astype(np.float64) @ di.bf16_to_f32(w).astype(np.float64).T
    # fp32 accumulation of exact bf16 products: error ~ sqrt(K) * eps_fp32 * |terms|
    np.testing.assert_allclose(c, ref, rtol=0, atol=1e-5 * np.sqrt(K) * np.abs(ref).max())


@pytest.mark.parametrize("M,F,K", [(7, 8200, 128), (70, 8192, 192), (200, 8256, 128), (272, 8192, 256), (320, 8960, 128), (301, 8960, 192), (330, 8448, 128),
                                   (530, 8192, 192), (1088, 8320, 128), (40, 96, 256), (300, 160, 128), (700, 256, 192)])
def test_gate_up_silu_epilogue_against_fp64(das, M, F, K):
    """silu(a Wg^T) * (a Wu^T) through the gate/up GEMM (every launch shape: wide outputs at 7 ... 1088 rows -- both tile heights of the 193..320-row range --, narrow ones)
    against fp64 on the same bf16 inputs; the kernel rounds its result to bf16."""
    rng = np.random.default_rng(M + F)
    a = di.f32_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    wg = di.f32_to_bf16(rng.standard_normal((F, K)).astype(np.float32) * 0.1)
    wu = di.f32_to_bf16(rng.standard_normal((F, K)).astype(np.float32) * 0.1)
    print(f"gate/up M={M} F={F} K={K}", flush=True)
    got = das.debug_gemm_silu(a, wg, wu)
    A = di.bf16_to_f32(a).astype(np.float64)
    g = A @ di.bf16_to_f32(wg).astype(np.float64).T
    u = A @ di.bf16_to_f32(wu).astype(np.float64).T
    ref = g / (1.0 + np.exp(-g)) * u
    # bf16 rounding of the result (2^-9 relative) plus fp32 accumulation and the fast reciprocal of the sigmoid
    np.testing.assert_allclose(got, ref, rtol=2.0 ** -8, atol=1e-5 * np.sqrt(K) * np.abs(ref).max())


@pytest.mark.parametrize("M,N,K", [(5, 16384, 128), (40, 16384, 128), (70, 16400, 128), (100, 16384, 128), (130, 16512, 128), (170, 16384, 128),
                                   (200, 16384, 128), (250, 16512, 128), (272, 16512, 128), (470, 16512, 128), (300, 16640, 192), (530, 16400, 128), (1088, 16384, 256)])
def test_row_maximum_epilogue_against_fp64(das, M, N, K):
    """The LM-head GEMM of a greedy pass keeps only the lowest column of each row's maximum: equal to the argmax of
    the fp64 product wherever its top two values are further apart than the fp32 accumulation error; planted ties
    (duplicated weight rows) must resolve to the lower column."""
    rng = np.random.default_rng(M + N)
    a = di.f32_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    w = di.f32_to_bf16(rng.standard_normal((N, K)).astype(np.float32) * 0.1)
    # planted exact ties that are the row maximum in most rows: columns 3 and N-7 carry the same large weight row,
    # columns 5000 and 5001 its negative
    big = di.f32_to_bf16(rng.standard_normal(K).astype(np.float32) * 2.0)
    w[3] = w[N - 7] = big
    w[5000] = w[5001] = big ^ np.uint16(0x8000)
    print(f"row max M={M} N={N} K={K}", flush=True)
    got = das.debug_gemm_rowmax(a, w)
    ref = di.bf16_to_f32(a).astype(np.float64) @ di.bf16_to_f32(w).astype(np.float64).T
    want = ref.argmax(axis=1)                                  # numpy: first maximum
    top2 = np.partition(ref, -2, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0] > 1e-4 * np.sqrt(K) * np.abs(ref).max()) | np.isin(want, [3, 5000])
    assert clear.sum() > 0.8 * M and np.isin(want, [3, 5000]).sum() > 0.5 * M
    np.testing.assert_array_equal(got[clear], want[clear])
    # rows the tolerance leaves open must still name a column whose value is within it of the maximum
    open_rows = np.nonzero(~clear)[0]
    assert np.all(ref[open_rows, got[open_rows]] >= ref[open_rows].max(axis=1) - 1e-4 * np.sqrt(K) * np.abs(ref).max())


@pytest.mark.parametrize("N,K,rows", [(320, 3584, 600), (192, 18944, 600), (16416, 1024, 600), (256, 960, 600), (2048, 16384, 600),
                                      (400, 16384, 1100), (2048, 16384, 2250), (2048, 16384, 3000), (4608, 3584, 1475), (1536, 8960, 600)])
def test_gemm_rows_do_not_depend_on_the_row_count(das, N, K, rows):
    """A row of the product is the same bits whether it is computed among 7, 70, 300, 600 or 2250 rows: narrow outputs
    sum K in slices whose layout and grouping depend on K alone, whichever kernel shape the row count selects (slices
    over workgroups, folded in registers, the two slice groups of a long K in two workgroups on 192- or 256-row tiles,
    or -- too many tiles for one round, 3000 rows -- grouped inside one workgroup; 256x128 tiles where those alone fit one round, 1475 rows x 4608 columns); wide outputs sum K in one pass at every row count."""
    rng = np.random.default_rng(N + K)
    a = di.f32_to_bf16(rng.standard_normal((rows, K)).astype(np.float32))
    w = di.f32_to_bf16(rng.standard_normal((N, K)).astype(np.float32) * 0.05)
    full = das.debug_gemm(a, w)
    for m in (7, 70, 150, 300, 520):      # (N = 2048, K = 16384 at 150 and 300 rows: all rows in one workgroup per column tile)
        print(f"gemm rows {m} of {rows}, N={N} K={K}", flush=True)
        part = das.debug_gemm(a[:m], w)
        assert np.array_equal(part, full[:m]), (m, float(np.abs(part - full[:m]).max()))


def _small_model(das, shape, **kw):
    args = dict(max_seqs=8, max_ctx=4096, max_rows=256, max_draft=8, num_pages=1024)
    args.update(kw)
    cfg = das.config_for(shape, **args)
    return das.DasModel(cfg, di.weights_bf16(shape, seed=0))


@pytest.mark.parametrize("model", ["tiny", "hd128"])
def test_kv_synth_import_export_are_bit_exact(das, model):
    shape = di.MODELS["tiny"] if model == "tiny" else di.MODELS["tiny"].replace(n_q_heads=6, n_kv_heads=2, head_dim=128, d_model=256)
    dm = _small_model(das, shape)
    ctx = 1000
    dm.seq_create(5, ctx, 3)
    print("kv_synth", model, flush=True)
    dm.kv_synth(5, seed=42, seq_key=9)
    for layer in range(shape.n_layers):
        k, v = dm.kv_export(5, layer, 0, ctx)
        np.testing.assert_array_equal(k, di.kv_synth(42, 9, layer, 0, 0, ctx, shape.n_kv_heads, shape.head_dim))
        np.testing.assert_array_equal(v, di.kv_synth(42, 9, layer, 1, 0, ctx, shape.n_kv_heads, shape.head_dim))
    # import a window, read it back, neighbours untouched
    # (any bf16 pattern with 2^-17 <= |x| < 2^16 minus one ulp: the range the pages hold exactly)
    rng = np.random.default_rng(0)

    def patterns():
        sh = (37, shape.n_kv_heads, shape.head_dim)
        e = rng.integers(127 - 17, 127 + 16, size=sh)
        m = rng.integers(0, 128, size=sh)
        m = np.where(e == 127 + 15, np.minimum(m, 126), m)          # 0x477F = 65280 is the largest bf16 below 65504
        return ((rng.integers(0, 2, size=sh) << 15) | (e << 7) | m).astype(np.uint16)
    kk, vv = patterns(), patterns()
    kk[0, 0, :4] = [0, 0x8000, 0x3F80, 0xBF80]                       # +-0, +-1
    dm.kv_import(5, 1, 100, kk, vv)
    k, v = dm.kv_export(5, 1, 90, 60)
    np.testing.assert_array_equal(k[10:47], kk)
    np.testing.assert_array_equal(v[10:47], vv)
    np.testing.assert_array_equal(k[:10], di.kv_synth(42, 9, 1, 0, 90, 10, shape.n_kv_heads, shape.head_dim))
    np.testing.assert_array_equal(v[47:], di.kv_synth(42, 9, 1, 1, 137, 13, shape.n_kv_heads, shape.head_dim))
    # outside that range: magnitudes above the binary16 maximum saturate at it (65504, which reads back as the bf16
    # next to it, 65536); magnitudes below 2^-17 move to a multiple of 2^-24 at most 3e-8 away
    edge = np.zeros((1, shape.n_kv_heads, shape.head_dim), np.float32)
    edge[0, 0, :6] = [1.0e6, -3.0e38, 65280.0, 2.0 ** -17, 1.0e-6, -2.0 ** -26]
    eb = di.f32_to_bf16(edge)
    dm.kv_import(5, 0, 200, eb, eb)
    k, v = dm.kv_export(5, 0, 200, 1)
    got = di.bf16_to_f32(k)[0, 0, :6]
    assert list(got[:4]) == [65536.0, -65536.0, 65280.0, 2.0 ** -17], got
    assert abs(got[4] - 1.0e-6) <= 3.0e-8 and got[5] == 0.0, got
    np.testing.assert_array_equal(k, v)
    dm.free()


def test_device_random_init_equals_the_host_blob(das):
    """das_model_load without a weight blob draws the N(0, 0.02^2) weights on the device from the seed with the same
    counter-based generator as das_inputs.weights_bf16: a model loaded either way gives the same bits (logits of a
    prefill and of a verify step, written KV)."""
    for shape in (di.MODELS["tiny"], di.MODELS["tiny"].replace(n_q_heads=6, n_kv_heads=2, head_dim=128, d_model=384, d_ffn=1000, vocab=20000)):
        cfg = das.config_for(shape, max_seqs=4, max_ctx=256, max_rows=64, max_draft=4, num_pages=64)
        prompts = di.prompts([19, 40], shape.vocab, 5)
        got = []
        for blob in (di.weights_bf16(shape, seed=3), None):
            dm = das.DasModel(cfg, blob, keep_logits=True, seed=3)
            nxt = dm.prefill([0, 1], prompts)
            l0 = dm.debug_logits()
            acc, nx = dm.verify_step([0, 1], [19, 40], [[5, 6, 7], [8]])
            got.append((nxt, l0, acc, nx, dm.debug_logits(), dm.kv_export(1, shape.n_layers - 1, 0, 41)))
            dm.free()
        a, b = got
        for x, y in zip(a[:5], b[:5]):
            assert np.array_equal(x, y)
        assert np.array_equal(a[5][0], b[5][0]) and np.array_equal(a[5][1], b[5][1])
    # a different seed is a different model
    dm = das.DasModel(cfg, None, keep_logits=True, seed=4)
    dm.prefill([0, 1], prompts)
    assert not np.array_equal(dm.debug_logits(), got[1][1])
    dm.free()


def test_kv_saturation_is_counted(das):
    """K/V pages hold bf16 values in binary16 containers: a value beyond +-65504 is stored saturated, and every such
    store is counted where the caller can read it -- from das_kv_import and from a pass that computes such values."""
    shape = di.MODELS["tiny"]
    blob = di.weights_bf16(shape, seed=0)
    cfg = das.config_for(shape, max_seqs=4, max_ctx=256, max_rows=64, max_draft=4, num_pages=64)
    dm = das.DasModel(cfg, blob)
    prompts = di.prompts([30], shape.vocab, 1)
    dm.prefill([0], prompts)
    dm.verify_step([0], [30], [[1, 2]])
    dm.kv_commit([0], [0], [7])
    assert dm.debug_kv_saturated() == 0
    k = np.zeros((3, shape.n_kv_heads, shape.head_dim), np.float32)
    v = np.zeros_like(k)
    k[0, 0, :2] = [70000.0, -1.0e9]
    v[2, 1, 5] = 3.0e38
    k[1, 0, 0] = 65280.0                                   # the largest bf16 below the container's maximum: not counted
    dm.kv_import(0, 1, 4, di.f32_to_bf16(k), di.f32_to_bf16(v))
    assert dm.debug_kv_saturated() == 3
    dm.free()
    # a model whose first input gain is 1e7 produces keys and values of the order 1e6 in layer 0
    hot = blob.copy()
    off = shape.vocab * shape.d_model
    hot[off:off + shape.d_model] = di.f32_to_bf16(np.full(shape.d_model, 1.0e7, np.float32))
    dm = das.DasModel(cfg, hot)
    dm.prefill([0], prompts)
    assert dm.debug_kv_saturated() > 100
    dm.free()
