"""Full-size parity of the bf16 workloads (medium, large, attn) in the launch configuration bench.py
times.  Expected values are digests written by tests/golden/make_digests.py, which calls only the
CPU oracle: loss, per-tensor gradient norms, the entries of every gradient tensor that
tests/golden/digest_index.py selects (a seeded sample, boundary rows, one 256 x 256 block per large
matrix), embedding-gradient rows of frequent and never-seen ids, per-position nll, and the first
positions of the forward intermediates.

The attn workload, the medium shape and two of the four networks of the paper's training-speed table
(well-conditioned initialisation) are also run with the paper's regularisation (dropout 0.2, label
smoothing 0.1) at the bar.

Three kinds of case:
  * bf16 path, bar of the task (loss rel 2e-2; gradients relative L2 <= 2e-2 and
    |g - g*| <= 2e-2 |g*| + 1e-3): the attn workload as specified, and the medium / large shapes
    with the parameters drawn at uniform[-0.05, 0.05).
  * fp32 path on the medium workload exactly as specified (uniform[-0.1, 0.1)): bar 1e-4.  This
    pins the schedule, indexing and tiling at the benchmark's shapes.
  * bf16 path on medium / large exactly as specified ("sens" mode).  At hidden size 1024 the
    [-0.1, 0.1) initialisation makes the recurrences chaotic: under the oracle's bf16 precision model
    (parameters and every contraction operand rounded to bfloat16, sums exact) the EXACT gradient moves
    by s = |g_bf16 - g| / |g| = 9-22 % per tensor at the medium workload and by about 100 % at the
    large one's 80 steps (tests/test_oracle_conditioning.py shows the effect on the CPU; the digest
    stores s per tensor, computed by the oracle alone).  No method
    whose operands are bf16 can be closer to g(W) than that, so here every gradient tensor is held to
    a bound RELATIVE TO ITS OWN SENSITIVITY: relative L2 error over the kept entries
    <= max(2e-2, SENS_C * s), and cosine with the oracle's entries >= 1 - (SENS_C * s)^2 / 2 - 1e-3
    (the cosine of two equally long vectors that far apart), and its norm to within SENS_C * s.
    Measured: at the medium workload every tensor is within 1.7 s (cosines 0.969-0.997 against
    0.988-0.996 for the oracle pair itself); at the large workload s is about 1 for everything but
    W_o / B_o — the exact gradient at bf16-rounded weights is itself uncorrelated with g(W)
    (cosines 0.36-0.66) — so there only W_o, B_o, the norms, the loss and the forward values carry
    information, and the gradient tiling at that shape is pinned by the 0.05-initialisation case.
    What the chaos does not reach is held at the plain bar: the loss, B_o, W_o where 2 s < 2e-2, and —
    in relative L2 — H_s at the first source positions and H_t / attention weights / context / H_o /
    nll of the first target positions (H_s and the attention weights also element by element)."""
import os
import sys

import numpy as np
import pytest

from paper_1802_07170_amd import inputs as I

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
sys.path.insert(0, GOLD)
import digest_index as DI  # noqa: E402

sample_index = DI.sample_index
SENS_C = 2.0


def kept_entries(d, key, k, v, shape):
    """(HIP path's entries, oracle's entries) of tensor k: the seeded sample plus the structured pieces."""
    got = [v[DI.sample_index(k, v.size)]]
    ref = [d[f"{key}/{k}"]]
    if key == "sample":
        for pn, piece in DI.pieces(shape).items():
            if f"piece/{pn}/{k}" in d:
                got.append(DI.take(v, shape, piece).reshape(-1))
                ref.append(d[f"piece/{pn}/{k}"].reshape(-1).astype(np.float64))
    return np.concatenate(got), np.concatenate(ref)


REG = dict(dropout=0.2, label_smoothing=0.1, dropout_seed=20180207)     # as in tests/golden/make_digests.py


def prefix_checks(tr, d, B, S, T, H, rtol, atol, report, mode):
    """Forward intermediates at the first positions (H_s at the first source positions; H_t, attention
    weights, context and H_o of the first decoder steps).  Every one of them is held to the relative-L2
    bar of the precision in every mode.  Element by element (|x - x*| <= rtol |x*| + atol) they are held
    in 'bar' mode; in 'sens' mode only H_s and the attention weights are: the decoder starts from the
    encoder's final states, which have been through all source positions of the chaotic recurrences, so
    its very first steps already carry absolute errors of 5e-3 to 1e-2 on single units (the same kernels
    stay below 4e-4 at the well-conditioned initialisation)."""
    Bp = tr.padded_batch()
    n_src, n_tgt = d["prefix/h_s"].shape[0], d["prefix/h_o"].shape[0]
    fetched = {"h_s": tr.debug_fetch("h_s", (S, Bp, H))[:n_src, :B], "h_t": tr.debug_fetch("h_t", (T, Bp, H))[:n_tgt, :B],
               "att_a": tr.debug_fetch("att_a", (T, Bp, S))[:n_tgt, :B], "att_cs": tr.debug_fetch("att_cs", (T, Bp, H))[:n_tgt, :B],
               "h_o": tr.debug_fetch("h_o", (T, Bp, H))[:n_tgt, :B]}
    for key, got in fetched.items():
        ref = d[f"prefix/{key}"].astype(np.float64)
        err = np.abs(got - ref)
        bound = rtol * np.abs(ref) + atol
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        report[f"prefix/{key}"] = (float(rel), float((err / bound).max()))
        assert rel <= rtol, f"prefix {key}: relative L2 {rel:.3e}"
        if mode == "bar" or key in ("h_s", "att_a"):
            assert (err <= bound).all(), f"prefix {key}: worst error {err.max():.3e}, {int((err > bound).sum())} entries outside the bound"


def run_digest_case(name, scale, prec, mode, reg=False):
    """mode: 'bar' = the tolerance of the precision; 'sens' = bounds relative to the oracle's own
    sensitivity to bf16-rounded parameters (see the module docstring).
    reg: the step with the paper's dropout and label smoothing."""
    from paper_1802_07170_amd import binding
    path = os.path.join(GOLD, f"digest_{name}" + (f"_s{scale}" if scale is not None else "") + ("_reg" if reg else "") + ".npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated")
    d = np.load(path)
    c = I.CONFIGS[name]
    cfg = I.model_cfg(c)
    params = I.make_params(cfg, c["seed"], 0.1 if scale is None else float(scale))
    batch = I.make_batch(c)
    B, S = batch[0].shape
    T = batch[2].shape[1]
    rtol, atol = (1e-4, None) if prec == 0 else (2e-2, 1e-3)
    tr = binding.Trainer(cfg, B, S, T, precision=prec)
    try:
        tr.set_params(I.flatten(params, cfg))
        if reg:
            tr.set_regularization(REG["dropout"], REG["label_smoothing"], REG["dropout_seed"])
        dev = tr.upload_batch(*batch)
        loss = tr.train_step(dev)
        flat = tr.get_grads()
        assert abs(loss - float(d["loss"])) <= rtol * float(d["loss"])
        g = I.unflatten(flat, cfg)
        report, lines = {}, []
        for k, shape in I.param_table(cfg):
            v = g[k].reshape(-1).astype(np.float64)
            assert np.isfinite(v).all(), k
            got, ref = kept_entries(d, "sample", k, v, shape)
            rel = np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-300)
            nrm, nref = np.linalg.norm(v), float(d[f"norm/{k}"])
            report[k] = rel
            s_k = float(d[f"sens/{k}"]) if mode == "sens" else 0.0
            if mode == "bar" or SENS_C * s_k <= rtol:
                bound = rtol * np.abs(ref) + (atol if atol is not None else rtol * np.abs(ref).max())
                bad = np.abs(got - ref) > bound
                assert not bad.any(), f"{k}: {bad.sum()} kept entries outside the bound"
                assert rel <= rtol, f"{k}: relative L2 over the kept entries {rel:.3e}"
                assert abs(nrm - nref) <= rtol * nref, k
            else:
                cos = float(got @ ref / (np.linalg.norm(got) * np.linalg.norm(ref) + 1e-300))
                cs = SENS_C * s_k
                lines.append(f"    {k:14s} s {s_k:.3f}  rel {rel:.3f} (<= {cs:.3f})  cos {cos:.4f} (>= {1 - cs * cs / 2 - 1e-3:.4f})  "
                             f"oracle pair: cos {float(d[f'cos_bf/{k}']):.4f}  |g|/|g*| {nrm / nref:.3f}")
                assert rel <= cs, f"{k}: relative L2 {rel:.3e} against {SENS_C} x sensitivity {s_k:.3e}"
                assert cos >= 1.0 - cs * cs / 2 - 1e-3, f"{k}: cosine {cos:.4f} with sensitivity {s_k:.3e}"
                assert abs(nrm - nref) <= cs * nref, (k, nrm, nref)
        for side in ("E_src", "E_tgt"):
            rows = d[f"rows_idx/{side}"]
            ref = d[f"rows/{side}"]
            got = g[side][rows].astype(np.float64)
            assert not got[16:].any() and not ref[16:].any()           # never-seen ids: exactly zero
            if mode == "bar":
                rel = np.linalg.norm(got[:16] - ref[:16]) / np.linalg.norm(ref[:16])
                assert rel <= rtol, (side, rel)
        Bp = tr.padded_batch()
        nll = tr.debug_fetch("nll", (T, Bp))[:, :B]
        ref = d["nll"]
        if mode == "bar":
            assert np.abs(nll - ref).max() <= (1e-4 if prec == 0 else 5e-2) * np.abs(ref).max()
        else:                                        # later positions drift with the chaotic forward pass: held on average
            assert np.abs(nll - ref).mean() <= 2e-2 * np.abs(ref).max()
            npre = d["prefix/h_o"].shape[0]
            assert np.abs(nll[:npre] - ref[:npre]).max() <= 2e-2 * np.abs(ref).max()
        assert not nll[ref == 0].any()
        if "prefix/h_s" in d:
            prefix_checks(tr, d, B, S, T, cfg["hidden"], rtol, atol if atol is not None else 1e-4, report, mode)
        # a second step gives bit-identical results (no atomics anywhere in the path)
        loss2 = tr.train_step(dev)
        assert loss2 == loss and np.array_equal(tr.get_grads(), flat)
        grads_only = {k: v for k, v in report.items() if not k.startswith("prefix/")}
        worst = max(grads_only, key=grads_only.get)
        print(f"\n{name} scale={scale or 0.1} prec={prec}: loss {loss:.6f} (oracle {float(d['loss']):.6f}); "
              f"worst relative L2 over the kept entries {report[worst]:.3e} ({worst}); W_o {report['W_o']:.3e}; "
              f"prefix relative L2 (worst error / element bound): "
              + ", ".join(f"{k[7:]} {v[0]:.1e} ({v[1]:.2f})" for k, v in report.items() if k.startswith("prefix/")))
        if lines:
            print("\n".join(lines))
    finally:
        tr.close()


def test_attn_workload_bf16_at_the_bar():
    run_digest_case("attn", None, 1, "bar")


@pytest.mark.parametrize("name", ["medium", "large"])
def test_h1024_shapes_bf16_well_conditioned_init_at_the_bar(name):
    run_digest_case(name, "0.05", 1, "bar")


def test_medium_workload_fp32_path_at_the_bar():
    run_digest_case("medium", None, 0, "bar")


def test_attn_workload_bf16_with_dropout_and_label_smoothing_at_the_bar():
    run_digest_case("attn", None, 1, "bar", reg=True)


def test_medium_shape_bf16_with_dropout_and_label_smoothing_at_the_bar():
    run_digest_case("medium", "0.05", 1, "bar", reg=True)


@pytest.mark.parametrize("name", ["paper_512x2", "paper_1024x4"])
def test_paper_speed_table_shapes_bf16_with_regularisation_at_the_bar(name):
    """The smallest and the largest network of the paper's training-speed table (vocabulary 37000: 578
    groups of 64 columns + 8), the step as the paper trains it (dropout 0.2, label smoothing 0.1)."""
    run_digest_case(name, "0.05", 1, "bar", reg=True)


@pytest.mark.parametrize("name", ["medium", "large"])
def test_h1024_workloads_bf16_as_specified(name):
    run_digest_case(name, None, 1, "sens")
