"""Seeded synthetic inputs for the training-step workloads.

This module holds no arithmetic of the method: it only draws token ids, sentence lengths and
parameter values, and lists tensor shapes.  Both the HIP path's tests / benchmark and the CPU
checker's tests take their inputs from here, so that they see the same numbers.

The workloads stand in for the paper's WMT English-German BPE data (Benchmarks, Settings; corpus
table): integer id matrices, ragged lengths padded per batch, a Zipf-like token distribution,
vocabularies of 32k-50k against the paper's ~37k, lengths bracketing the corpus mean of ~25.
"""
from __future__ import annotations

import numpy as np

PAD_ID, BOS_ID = 0, 2

# name -> model + batch recipe.  "precision": 0 = fp32 path, 1 = bf16-MFMA path.
CONFIGS = {
    "tiny":   dict(src_vocab=1000, tgt_vocab=1000, emb=64, hidden=64, layers=1, precision=0,
                   batch=8, len_range=(10, 10), ids="uniform", seed=0),
    "small":  dict(src_vocab=32000, tgt_vocab=32000, emb=512, hidden=512, layers=2, precision=0,
                   batch=64, len_range=(10, 50), ids="zipf", seed=1),
    "medium": dict(src_vocab=32000, tgt_vocab=32000, emb=1024, hidden=1024, layers=4, precision=1,
                   batch=64, len_range=(20, 50), ids="zipf", seed=2),
    "large":  dict(src_vocab=50000, tgt_vocab=50000, emb=1024, hidden=1024, layers=4, precision=1,
                   batch=128, len_range=(30, 80), ids="zipf", seed=3),
    "attn":   dict(src_vocab=32000, tgt_vocab=32000, emb=512, hidden=512, layers=2, precision=1,
                   batch=32, len_range=(120, 120), ids="zipf", seed=4),
}
# The four networks of the paper's training-speed table (embedding = hidden size 512 or 1024, 2 or 4
# layers on each side), with its vocabulary of about 37000.  The paper does not state its batch size:
# 64 sentences here; lengths uniform in [5, 45] (mean 25, the corpus table's tokens per sentence).
for _h in (512, 1024):
    for _l in (2, 4):
        CONFIGS[f"paper_{_h}x{_l}"] = dict(src_vocab=37000, tgt_vocab=37000, emb=_h, hidden=_h, layers=_l, precision=1,
                                           batch=64, len_range=(5, 45), ids="zipf", seed=10 + _h // 512 + _l)
PAPER_SHAPES = [k for k in CONFIGS if k.startswith("paper_")]


def model_cfg(c):
    return {k: c[k] for k in ("src_vocab", "tgt_vocab", "emb", "hidden", "layers")}


def param_table(cfg):
    """Canonical flat parameter order: list of (name, shape), row-major [out, in]."""
    Vs, Vt, E, H, L = cfg["src_vocab"], cfg["tgt_vocab"], cfg["emb"], cfg["hidden"], cfg["layers"]
    Hd = H // 2
    t = [("E_src", (Vs, E)), ("E_tgt", (Vt, E))]
    for d in ("fwd", "bwd"):
        t += [(f"enc.l0.{d}.W", (4 * Hd, E + Hd)), (f"enc.l0.{d}.b", (4 * Hd,))]
    for l in range(1, L):
        t += [(f"enc.l{l}.W", (4 * H, 2 * H)), (f"enc.l{l}.b", (4 * H,))]
    t += [("dec.l0.W", (4 * H, E + 2 * H)), ("dec.l0.b", (4 * H,))]
    for l in range(1, L):
        t += [(f"dec.l{l}.W", (4 * H, 2 * H)), (f"dec.l{l}.b", (4 * H,))]
    t += [("W_a", (H, H)), ("W_c", (H, 2 * H)), ("W_o", (Vt, H)), ("B_o", (Vt,))]
    return t


def param_count(cfg):
    return int(sum(int(np.prod(s)) for _, s in param_table(cfg)))


def make_params(cfg, seed, scale=0.1):
    """float32 parameters, uniform[-scale, scale), as a dict in canonical order."""
    rng = np.random.default_rng([seed, 7])
    return {name: rng.uniform(-scale, scale, size=shape).astype(np.float32)
            for name, shape in param_table(cfg)}


def flatten(params, cfg):
    return np.concatenate([np.asarray(params[n], np.float32).reshape(-1) for n, _ in param_table(cfg)])


def unflatten(flat, cfg):
    out, o = {}, 0
    for name, shape in param_table(cfg):
        n = int(np.prod(shape))
        out[name] = np.asarray(flat[o:o + n]).reshape(shape)
        o += n
    return out


def zipf_ids(rng, vocab, size, s=1.1):
    """Bounded Zipf law p(rank k) ~ k^-s for k = 1..vocab-4, id = 3 + k (ids in [4, vocab)),
    sampled by inverse CDF."""
    k = np.arange(1, vocab - 3, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    r = np.searchsorted(cdf, rng.random(size), side="left")
    return (4 + np.minimum(r, vocab - 5)).astype(np.int32)


def make_batch(c, batch=None, len_range=None, seed=None):
    """Draws, in this order: src_len, tgt_len, src_ids, tgt_ids.  S, T = the batch maxima;
    padded slots hold PAD_ID.  Returns int32 arrays src_ids [B,S], src_len [B], tgt_ids [B,T],
    tgt_len [B]."""
    B = c["batch"] if batch is None else batch
    lo, hi = c["len_range"] if len_range is None else len_range
    rng = np.random.default_rng(c["seed"] if seed is None else seed)
    src_len = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    tgt_len = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    S, T = int(src_len.max()), int(tgt_len.max())
    if c["ids"] == "uniform":
        src = rng.integers(4, c["src_vocab"], size=(B, S)).astype(np.int32)
        tgt = rng.integers(4, c["tgt_vocab"], size=(B, T)).astype(np.int32)
    else:
        src = zipf_ids(rng, c["src_vocab"], (B, S))
        tgt = zipf_ids(rng, c["tgt_vocab"], (B, T))
    src[np.arange(S)[None, :] >= src_len[:, None]] = PAD_ID
    tgt[np.arange(T)[None, :] >= tgt_len[:, None]] = PAD_ID
    return src, src_len, tgt, tgt_len
