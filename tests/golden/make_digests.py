"""Writes the expected values for the full-size parity tests of the three bf16 workloads
(medium, large, attn).  Calls only the CPU oracle (oracle/) on the seeded inputs; nothing here
comes from the HIP path.

    python tests/golden/make_digests.py [medium large attn medium:0.05 large:0.05 attn::reg medium:0.05:reg
                                          paper_512x2:0.05:reg paper_1024x4:0.05:reg]

A name with ":scale" draws the same parameters at uniform[-scale, scale) instead of the workload's
[-0.1, 0.1): at hidden size 1024 the 0.1 initialisation makes the recurrences chaotic (rounding
the weights to bf16 alone moves the exact gradient by 15-30 %), so the bf16 path is also checked
at the full shapes with a well-conditioned initialisation.  A third field "reg" runs the step with
the paper's regularisation: dropout 0.2, label smoothing 0.1 (mask seed REG_SEED).

Per workload a compressed .npz with: the loss, the per-tensor L2 norm and max|g| of every gradient,
a seeded sample of 4096 entries per gradient tensor (all entries of tensors up to 65536 elements),
the embedding rows of the 16 most frequent and of 16 never-seen token ids, and per-position nll.
Runs for a few minutes on 8 cores (the large workload needs ~20 GB of memory)."""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import nmt_oracle as O  # noqa: E402
from paper_1802_07170_amd import inputs as I  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
SAMPLE = 4096
SMALL = 65536
REG = dict(dropout=0.2, label_smoothing=0.1, dropout_seed=20180207)


def sample_index(name, n):
    """The same seeded sample positions are drawn by the test."""
    if n <= SMALL:
        return np.arange(n)
    seed = int.from_bytes(name.encode(), "little") % (2 ** 31)
    return np.sort(np.random.default_rng(seed).choice(n, size=SAMPLE, replace=False))


def main():
    names = sys.argv[1:] or ["medium", "large", "attn", "medium:0.05", "large:0.05"]
    for spec in names:
        name, sc, reg = (spec.split(":") + ["", ""])[:3]
        scale = float(sc) if sc else 0.1
        kw = REG if reg == "reg" else {}
        c = I.CONFIGS[name]
        cfg = I.model_cfg(c)
        params = I.make_params(cfg, c["seed"], scale)
        batch = I.make_batch(c)
        t0 = time.time()
        loss, g, it = O.train_step(cfg, params, *batch, want_intermediates=True, **kw)
        out = {"loss": np.float64(loss), "oracle_seconds": np.float64(time.time() - t0),
               "nll": it["nll"].astype(np.float32)}
        for k, v in g.items():
            flat = v.reshape(-1)
            out[f"norm/{k}"] = np.float64(np.linalg.norm(flat))
            out[f"max/{k}"] = np.float64(np.abs(flat).max())
            out[f"sample/{k}"] = flat[sample_index(k, flat.size)].astype(np.float64)
        for side, ids in (("E_src", batch[0]), ("E_tgt", batch[2])):
            cnt = np.bincount(ids.reshape(-1), minlength=cfg["src_vocab"])
            top = np.argsort(-cnt)[:16]
            unseen = np.where(cnt == 0)[0]
            unseen = unseen[unseen >= 4][:16]
            rows = np.concatenate([top, unseen])
            out[f"rows_idx/{side}"] = rows.astype(np.int64)
            out[f"rows/{side}"] = g[side][rows].astype(np.float64)
        path = os.path.join(HERE, f"digest_{name}" + (f"_s{sc}" if sc else "") + ("_reg" if kw else "") + ".npz")
        np.savez_compressed(path, **out)
        print(f"{name}: loss {loss:.6f}, {time.time() - t0:.1f} s -> {path} ({os.path.getsize(path) / 1e6:.1f} MB)", flush=True)


if __name__ == "__main__":
    main()
