"""The entry point that allocates nothing (das_gemm_noalloc) against the one it is a variant of (das_debug_gemm)."""
import numpy as np
import pytest

import das_inputs as di

pytestmark = pytest.mark.gpu


def test_gemm_noalloc_equals_debug_gemm_on_two_calls_in_a_row():
    import torch
    import paper_2511_13841_amd as das
    rng = np.random.default_rng(11)
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    # the second call is smaller in every dimension: nothing of the first may leak into it through the shared array
    for (M, N, K) in [(250, 2000, 2048), (70, 520, 136)]:
        a = di.f32_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
        w = di.f32_to_bf16(rng.standard_normal((N, K)).astype(np.float32) * 0.05)
        a_d = torch.from_numpy(a.view(np.int16)).to(dev)
        w_d = torch.from_numpy(w.view(np.int16)).to(dev)
        c_d = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        print(f"gemm_noalloc M={M} N={N} K={K}", flush=True)
        das.gemm_noalloc(M, N, K, a_d.data_ptr(), w_d.data_ptr(), c_d.data_ptr(), stream)
        torch.cuda.synchronize()
        got = c_d.cpu().numpy()
        want = das.debug_gemm(a, w)
        assert np.array_equal(got, want), float(np.abs(got - want).max())
        ref = di.bf16_to_f32(a).astype(np.float64) @ di.bf16_to_f32(w).astype(np.float64).T
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-5 * np.sqrt(K) * np.abs(ref).max())
    # beyond the stated maximum: a clear error, nothing launched
    with pytest.raises(das.DasError) as e:
        das.gemm_noalloc(257, 64, 64, a_d.data_ptr(), w_d.data_ptr(), c_d.data_ptr(), stream)
    assert e.value.code == das.DAS_ERR_INVALID
    with pytest.raises(das.DasError):
        das.gemm_noalloc(16, 64, 4096, a_d.data_ptr(), w_d.data_ptr(), c_d.data_ptr(), stream)
