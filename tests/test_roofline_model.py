"""The intensity calculator reproduces the numbers the paper prints (appendix "Arithmetic
Intensity Analysis") and its closed forms."""
import os

import numpy as np

from paper_2511_16652_amd import roofline

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "arithmetic_intensity.txt")


def test_critical_batches_printed_in_the_paper():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert rows
    for m, A, r, std, egg in rows:
        m, A, r = int(m), float(A), int(r)
        assert roofline.critical_batch_standard(A, m) == int(std)
        assert roofline.critical_batch_eggroll(A, m, r) == int(egg)
        # the critical batch really is where the general formulas cross A
        assert roofline.intensity_standard(int(std), m, m) >= A > roofline.intensity_standard(int(std) - 1, m, m)
        assert roofline.intensity_eggroll(int(egg), m, m, r) >= A > roofline.intensity_eggroll(int(egg) - 1, m, m, r)


def test_closed_forms():
    m, B = 8192, 1024
    assert np.isclose(roofline.intensity_standard(B, m, m), B * m / (2.0 * B + m))
    assert np.isclose(roofline.intensity_gaussian_es(m, m), m / (2.0 + m))
    assert roofline.intensity_gaussian_es(m, m) < 1.0
    r = 1
    extra = roofline.forward_flops(B, m, m, r) - 2.0 * B * m * m
    assert np.isclose(extra, B * m * (4 * r + 1))
    assert np.isclose(extra / (2.0 * B * m * m), roofline.flop_overhead(r, m))
