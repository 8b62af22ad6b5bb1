"""The seeded input generators: what the tests and the benchmark rely on (no method arithmetic here)."""
import numpy as np

import workloads as WL


def test_logit_bias_spreads_routes_evenly_and_is_reproducible():
    a = WL.seeded_logit_bias(11, 256, 14)
    b = WL.seeded_logit_bias(11, 256, 14)
    assert np.array_equal(a, b) and a.dtype == np.float32 and a.shape == (256, 14)
    hist = np.bincount(a.argmax(1), minlength=14)
    assert hist.min() >= 18 and hist.max() <= 19          # 256 = 14 * 18 + 4
    top2 = np.sort(a, axis=1)[:, -2:]
    assert np.all(top2[:, 1] - top2[:, 0] > 3.0)          # margins far above rounding noise


def test_skewed_logit_bias_puts_half_of_the_batch_on_one_route():
    T, B = 4, 256
    for favour in (0, T - 1):
        a = WL.seeded_logit_bias(5, B, T, amp=16.0, favour=favour)
        hist = np.bincount(a.argmax(1), minlength=T)
        assert hist.sum() == B
        assert hist[favour] == B // 2 + B // 2 // T       # the favoured half plus its share of the spread half
        others = np.delete(hist, favour)
        assert others.min() == others.max() == B // 2 // T
    # the default draw is untouched by the extra arguments
    assert np.array_equal(WL.seeded_logit_bias(5, B, T, amp=16.0), WL.seeded_logit_bias(5, B, T, amp=16.0, favour=-1))


def test_images_and_bf16_rounding_are_deterministic():
    x = WL.images(3, 2, size=32)
    assert x.shape == (2, 3, 32, 32) and np.array_equal(x, WL.images(3, 2, size=32))
    r = WL.nets.as_bf16_values(x)
    assert np.array_equal(r, x)                           # already bf16-representable
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
