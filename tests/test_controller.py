"""The learning-rate rule of the paper's training procedure (section "Comparison on Translation
Quality"), on hand-made entropy sequences."""
import math

import pytest

from paper_1802_07170_amd import controller as C


def test_improvement_needs_the_margin_and_patience_counts_checks():
    c = C.LearningRateController(learning_rate=1.0)
    assert c.observe(5.0) == C.NEW_BEST
    assert c.margin() == 0.01                                   # max(0.01 * 1.0, 0.001)
    assert c.observe(4.995) == C.CONTINUE                       # better, but by less than the margin
    assert c.best == 5.0
    assert c.observe(4.98) == C.NEW_BEST and c.checks_without_improvement == 0
    for i in range(11):
        assert c.observe(4.98) == C.CONTINUE
    assert c.observe(4.975) == C.DECAY_AND_RESTART              # 12th check without improvement
    assert c.learning_rate == pytest.approx(0.7) and c.decays == 1 and c.best == 4.98
    assert c.margin() == pytest.approx(0.007)


def test_margin_floor_and_stop_rule():
    c = C.LearningRateController(learning_rate=0.05, patience=3)
    assert c.margin() == 0.001                                  # 0.01 * 0.05 < 0.001
    assert c.observe(3.0) == C.NEW_BEST
    assert [c.observe(3.0) for _ in range(3)] == [C.CONTINUE, C.CONTINUE, C.DECAY_AND_RESTART]
    assert c.observe(2.9) == C.NEW_BEST                         # improvement after the first decay
    assert [c.observe(2.9) for _ in range(3)] == [C.CONTINUE, C.CONTINUE, C.DECAY_AND_RESTART]
    assert c.decays == 2 and c.learning_rate == pytest.approx(0.05 * 0.49)
    # no improvement at all between the second decay and the next one that would be due: stop
    assert [c.observe(2.9) for _ in range(3)] == [C.CONTINUE, C.CONTINUE, C.STOP]
    assert c.observe(1.0) == C.STOP and c.stopped


def test_nan_never_improves_and_arguments_are_checked():
    c = C.LearningRateController(patience=2)
    assert c.observe(float("nan")) == C.CONTINUE and math.isinf(c.best)
    assert c.observe(2.0) == C.NEW_BEST
    with pytest.raises(ValueError):
        C.LearningRateController(decay=1.0)
    with pytest.raises(ValueError):
        C.LearningRateController(patience=0)
