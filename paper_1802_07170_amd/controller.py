"""Learning-rate control of the paper's training procedure (section "Comparison on Translation
Quality"; hyperparameter table: learning rate 1.0, decay 0.7): the development-set cross-entropy is
checked at regular intervals; when it has not improved by max(0.01 * learning_rate, 0.001) in 12
consecutive checks the learning rate is multiplied by 0.7 and training restarts from the best
parameters seen so far; training ends when a whole period between two neighbouring decays brought
no improvement.

Host logic only: it decides, the caller acts (runs steps with `Trainer.sgd_update(lr)`, keeps a copy
of the best parameters via `Trainer.get_params()` and puts it back with `Trainer.set_params()`)."""
from __future__ import annotations

CONTINUE, NEW_BEST, DECAY_AND_RESTART, STOP = "continue", "new_best", "decay_and_restart", "stop"


class LearningRateController:
    def __init__(self, learning_rate=1.0, decay=0.7, patience=12, relative_margin=0.01, margin_floor=0.001):
        if not (0.0 < decay < 1.0) or patience < 1 or learning_rate <= 0.0:
            raise ValueError("need 0 < decay < 1, patience >= 1, learning_rate > 0")
        self.learning_rate = float(learning_rate)
        self.decay = float(decay)
        self.patience = int(patience)
        self.relative_margin = float(relative_margin)
        self.margin_floor = float(margin_floor)
        self.best = float("inf")          # best development entropy so far (the model to restart from)
        self.checks_without_improvement = 0
        self.improved_since_last_decay = False
        self.decays = 0
        self.stopped = False

    def margin(self):
        return max(self.relative_margin * self.learning_rate, self.margin_floor)

    def observe(self, dev_entropy):
        """One development-set check.  Returns NEW_BEST (keep a copy of the parameters), CONTINUE,
        DECAY_AND_RESTART (self.learning_rate is already the decayed one; reload the best parameters)
        or STOP."""
        if self.stopped:
            return STOP
        x = float(dev_entropy)
        if x < self.best - self.margin():          # also true for the first finite value; NaN never improves
            self.best = x
            self.checks_without_improvement = 0
            self.improved_since_last_decay = True
            return NEW_BEST
        self.checks_without_improvement += 1
        if self.checks_without_improvement < self.patience:
            return CONTINUE
        # a decay is due: was there any improvement since the previous one?
        if self.decays > 0 and not self.improved_since_last_decay:
            self.stopped = True
            return STOP
        self.learning_rate *= self.decay
        self.decays += 1
        self.checks_without_improvement = 0
        self.improved_since_last_decay = False
        return DECAY_AND_RESTART
