"""The host-side schedules against the constants the paper prints (tests/golden/section4_schedules.txt)."""
import math
import os

import pytest

from paper_2010_02838_amd import schedules as S


def golden():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "section4_schedules.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = tuple(float(v) for v in line[1:])
    return out


def test_constants_are_the_printed_ones():
    g = golden()
    assert set(g) == set(S.PAPER)
    for k, v in g.items():
        have = S.PAPER[k] if isinstance(S.PAPER[k], tuple) else (S.PAPER[k],)
        assert tuple(float(x) for x in have) == v, k


def test_imagenet_schedules_at_the_printed_epochs():
    g = golden()
    ipe = 100                                                    # updates per epoch of this toy run
    peak = S.linear_scaled_lr(512)                               # two models x 256
    assert peak == pytest.approx(0.2)
    ms = [int(e) * ipe for e in g["lr_milestone_epochs_codistillation"]]
    lr = S.warmup_step_lr(peak, 5 * ipe, ms, g["lr_decay_factor"][0])
    assert lr(0) == pytest.approx(0.02) and lr(5 * ipe) == peak and lr(250) == pytest.approx(0.02 + 0.18 * 0.5)
    for e, scale in ((17, 1), (18, 0.1), (37, 0.1), (38, 0.01), (43, 0.01), (44, 0.001), (89, 0.001)):
        assert lr(e * ipe) == pytest.approx(peak * scale), e
    wd = S.stepped_l2(g["l2_initial_main_text"][0], ms)
    assert [wd(e * ipe) for e in (0, 17, 18, 37, 38, 44, 89)] == [5e-4, 5e-4, 1e-5, 1e-5, 0.0, 0.0, 0.0]
    cos = S.half_cosine_lr(peak, 5 * ipe, 90 * ipe)
    assert cos(5 * ipe) == peak and cos(90 * ipe) == pytest.approx(0.0, abs=1e-12)
    assert cos((5 * ipe + 90 * ipe) // 2) == pytest.approx(peak / 2, rel=1e-2)
    assert all(cos(k) >= cos(k + 1) for k in range(5 * ipe, 90 * ipe))


def test_translation_alpha_growth():
    g = golden()
    alpha = S.geometric(1.0, g["alpha_growth_per_epoch_translation"][0], 50)
    assert alpha(0) == 1.0 and alpha(49) == 1.0 and alpha(50) == pytest.approx(1.1) and alpha(175) == pytest.approx(1.1 ** 3)
    smooth = S.geometric(0.1, 0.5, 50)                           # label smoothing decayed over training
    assert smooth(100) == pytest.approx(0.025) and math.isclose(smooth(0), 0.1)
