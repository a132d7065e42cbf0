"""The paper's training procedure around the device step (Settings section and the hyperparameter
table; section "Comparison on Translation Quality" for the schedule): SGD on mini-batches with
dropout and label smoothing, the development-set cross-entropy checked at regular intervals, the
learning rate decayed and the best parameters restored when it stalls, and checkpoint files.

Host logic only.  Every number comes from the device library through `binding.Trainer`
(`train_step_async`, `sgd_update`, `eval_loss`, `get_params` / `set_params`); nothing here computes
any part of the model."""
from __future__ import annotations

import json

import numpy as np

from . import controller as C

CHECKPOINT_FORMAT = 1


def save_checkpoint(path, trainer, model_cfg, ctl=None, step=0):
    """One .npz file: the flat fp32 parameter vector in the library's canonical order, the tensor table
    it was written with (names, shapes, offsets), the model configuration, and the controller's state."""
    table = trainer.param_table()
    meta = {
        "format": CHECKPOINT_FORMAT,
        "model": {k: int(model_cfg[k]) for k in ("src_vocab", "tgt_vocab", "emb", "hidden", "layers")},
        "table": [[n, int(r), int(c), int(o)] for n, r, c, o in table],
        "step": int(step),
        "controller": None if ctl is None else {k: getattr(ctl, k) for k in (
            "learning_rate", "decay", "patience", "relative_margin", "margin_floor", "best",
            "checks_without_improvement", "improved_since_last_decay", "decays", "stopped")},
    }
    with open(path, "wb") as f:
        np.savez(f, params=trainer.get_params(), meta=np.frombuffer(json.dumps(meta).encode(), dtype=np.uint8))


def load_checkpoint(path, trainer, model_cfg, ctl=None):
    """Puts a checkpoint's parameters into the trainer (and its controller state into `ctl`).  The file
    must have been written for the same model: configuration and tensor table are compared.
    Returns the step count stored in the file."""
    with np.load(path, allow_pickle=False) as z:
        flat = np.ascontiguousarray(z["params"], dtype=np.float32)
        meta = json.loads(bytes(z["meta"]).decode())
    if meta.get("format") != CHECKPOINT_FORMAT:
        raise ValueError(f"{path}: unknown checkpoint format {meta.get('format')!r}")
    want = {k: int(model_cfg[k]) for k in ("src_vocab", "tgt_vocab", "emb", "hidden", "layers")}
    if meta["model"] != want:
        raise ValueError(f"{path}: written for model {meta['model']}, the trainer has {want}")
    table = [[n, int(r), int(c), int(o)] for n, r, c, o in trainer.param_table()]
    if meta["table"] != table:
        raise ValueError(f"{path}: the tensor table differs from the library's")
    if flat.size != trainer.n_params:
        raise ValueError(f"{path}: {flat.size} parameters, the trainer has {trainer.n_params}")
    trainer.set_params(flat)
    if ctl is not None and meta["controller"] is not None:
        for k, v in meta["controller"].items():
            setattr(ctl, k, v)
    return meta["step"]


def dev_entropy(trainer, dev_batches):
    """Cross-entropy per target token over a list of device batches, in evaluation mode."""
    total, count = 0.0, 0.0
    for b in dev_batches:
        loss, ntok = trainer.eval_loss(b)
        total += float(loss) * float(ntok)
        count += float(ntok)
    if count == 0:
        raise ValueError("the development set holds no target token")
    return total / count


def fit(trainer, train_batches, dev_batches, ctl, eval_every, max_steps, dropout=0.2, label_smoothing=0.1,
        seed=0, on_check=None):
    """Runs the schedule: `train_batches` (a sequence of device batches, cycled) feeds SGD steps at
    the controller's learning rate, each with its own dropout mask seed; every `eval_every` steps the
    development entropy goes to the controller, which keeps / decays / stops.  The best parameters are
    kept on the host and restored at every decay and at the end.
    Returns a list of (step, development entropy, learning rate used so far, action)."""
    if eval_every < 1 or max_steps < 1 or len(train_batches) == 0:
        raise ValueError("need eval_every >= 1, max_steps >= 1 and at least one training batch")
    history = []
    best = None
    step = 0
    while step < max_steps and not ctl.stopped:
        trainer.set_regularization(dropout, label_smoothing, seed + step)
        trainer.train_step_async(train_batches[step % len(train_batches)])
        trainer.sgd_update(ctl.learning_rate)
        step += 1
        if step % eval_every and step != max_steps:
            continue
        trainer.fetch_loss()                       # raises on a range / non-finite error of the last step
        lr = ctl.learning_rate
        entropy = dev_entropy(trainer, dev_batches)
        action = ctl.observe(entropy)
        if action == C.NEW_BEST:
            best = trainer.get_params()
        elif action == C.DECAY_AND_RESTART and best is not None:
            trainer.set_params(best)
        history.append((step, entropy, lr, action))
        if on_check is not None:
            on_check(step, entropy, lr, action)
    if best is not None:
        trainer.set_params(best)
    return history
