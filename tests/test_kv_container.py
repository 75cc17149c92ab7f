"""The KV pages hold bf16-rounded values in IEEE binary16 containers (include/das.h, das_kv_import).  This checks
the claimed value range on the CPU, over every bf16 bit pattern, with numpy's own conversions: which values survive
the round trip bf16 -> binary16 -> bf16 bit for bit, and how far the others move."""
import numpy as np

import das_inputs as di


def test_every_bf16_value_in_the_documented_range_survives_a_binary16_container():
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    x = di.bf16_to_f32(bits)
    finite = np.isfinite(x)
    # what the device does: clamp to the largest binary16 value, round to nearest even, widen, round to bf16
    with np.errstate(over="ignore"):
        h = np.clip(x, -65504.0, 65504.0).astype(np.float16)
    back = di.f32_to_bf16(h.astype(np.float32))
    a = np.abs(x)
    exact_range = finite & ((a == 0) | ((a >= 2.0 ** -17) & (a <= 65280.0)))
    assert exact_range.sum() == 33 * 128 * 2 + 2                       # 33 binades x 128 mantissas x 2 signs, and +-0
    np.testing.assert_array_equal(back[exact_range], bits[exact_range])
    # below the range: a multiple of 2^-24 at most 3e-8 away
    small = finite & (a > 0) & (a < 2.0 ** -17)
    moved = np.abs(h[small].astype(np.float64) - x[small].astype(np.float64))
    assert moved.max() <= 2.0 ** -25 + 1e-12 and moved.max() <= 3e-8
    # above it: saturation at 65504, which reads back as the bf16 next to it
    big = finite & (a > 65280.0)
    assert np.all(np.abs(h[big].astype(np.float32)) == 65504.0)
    assert np.all(np.abs(di.bf16_to_f32(back[big])) == 65536.0)
    # 65280 = 0x477F is the largest bf16 value below the binary16 maximum
    assert di.bf16_to_f32(np.array([0x477F], np.uint16))[0] == 65280.0
