"""The learning-rate rule of the paper's training procedure (section "Comparison on Translation
Quality"), on hand-made entropy sequences."""
import math

import numpy as np

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


class _StubTrainer:
    """Stands in for binding.Trainer: a parameter vector that each step moves towards a target, and a
    development loss that is the squared distance to it (so the host loop has something to steer)."""

    def __init__(self, n=6):
        self.n_params = n
        self.p = np.zeros(n, np.float32)
        self.target = np.arange(n, dtype=np.float32)
        self.reg = None
        self.calls = []

    def param_table(self):
        return [("a", 2, 2, 0), ("b", 2, 1, 4)]

    def get_params(self):
        return self.p.copy()

    def set_params(self, flat):
        self.calls.append("set")
        self.p = np.array(flat, np.float32)

    def set_regularization(self, dropout, ls, seed):
        self.reg = (dropout, ls, seed)

    def train_step_async(self, batch):
        self.calls.append(("step", batch, self.reg[2]))

    def fetch_loss(self):
        return 0.0

    def sgd_update(self, lr):
        self.p = (self.p + np.float32(0.5 * lr) * (self.target - self.p)).astype(np.float32)

    def eval_loss(self, batch):
        return float(((self.p - self.target) ** 2).sum()) + 0.25 * batch, 10.0 * (batch + 1)


def test_host_loop_cycles_batches_seeds_masks_and_weights_the_dev_average():
    from paper_1802_07170_amd import training as TR
    t = _StubTrainer()
    assert TR.dev_entropy(t, [0, 1]) == pytest.approx((55.0 * 10 + 55.25 * 20) / 30)
    ctl = C.LearningRateController(patience=2)
    hist = TR.fit(t, [0, 1, 2], [0, 1], ctl, eval_every=2, max_steps=7, dropout=0.2, label_smoothing=0.1, seed=40)
    steps = [c for c in t.calls if c != "set"]
    assert [b for _, b, _ in steps] == [0, 1, 2, 0, 1, 2, 0]          # batches cycled
    assert [s for _, _, s in steps] == list(range(40, 47))             # one mask seed per step
    assert [h[0] for h in hist] == [2, 4, 6, 7]                        # every 2 steps, and at the end
    assert all(h[3] == C.NEW_BEST for h in hist)
    assert t.reg[:2] == (0.2, 0.1)
    with pytest.raises(ValueError):
        TR.fit(t, [], [0], ctl, 1, 1)


def test_host_loop_restores_the_best_parameters_on_decay_and_at_the_end():
    from paper_1802_07170_amd import training as TR
    t = _StubTrainer()
    t.sgd_update = lambda lr: setattr(t, "p", (t.p + np.float32(1.0)).astype(np.float32))   # overshoots after a while
    ctl = C.LearningRateController(patience=2)
    hist = TR.fit(t, [0], [0], ctl, eval_every=1, max_steps=40)
    best_step = min(hist, key=lambda h: h[1])
    assert any(h[3] == C.DECAY_AND_RESTART for h in hist) and hist[-1][3] == C.STOP and ctl.stopped
    assert t.eval_loss(0)[0] == pytest.approx(best_step[1])            # best parameters in place at the end
    assert "set" in t.calls


def test_checkpoint_round_trip_and_mismatch(tmp_path):
    from paper_1802_07170_amd import training as TR
    cfg = dict(src_vocab=8, tgt_vocab=9, emb=2, hidden=2, layers=1)
    t = _StubTrainer()
    t.p = np.array([0.1, -2.5, 3e-8, 7, 1e30, -0.0], np.float32)
    ctl = C.LearningRateController(learning_rate=0.49, patience=5)
    ctl.observe(3.25); ctl.observe(3.3)
    path = tmp_path / "c.npz"
    TR.save_checkpoint(path, t, cfg, ctl, step=123)
    u = _StubTrainer()
    ctl2 = C.LearningRateController()
    assert TR.load_checkpoint(path, u, cfg, ctl2) == 123
    assert u.p.tobytes() == t.p.tobytes()                               # bit for bit, the sign of zero included
    assert vars(ctl2) == vars(ctl)
    with pytest.raises(ValueError):
        TR.load_checkpoint(path, u, dict(cfg, hidden=4))
    u.param_table = lambda: [("a", 2, 2, 0), ("b", 1, 2, 4)]
    with pytest.raises(ValueError):
        TR.load_checkpoint(path, u, cfg)
