"""cmt_eval_loss_static (the entry point that allocates nothing: every intermediate lives in a static
device array of the library) against cmt_eval_loss (intermediates in the caller's workspace): same
kernels in the same order, so the loss must be bit-identical and the token count equal — on two
calls in a row, the second with a smaller input, in both precisions; a shape whose intermediates do
not fit the array is refused with a clear message and leaves the handle usable."""
import numpy as np
import pytest

from paper_1802_07170_amd import inputs as I

pytestmark = pytest.mark.gpu


def _case(prec):
    from paper_1802_07170_amd import binding
    c = I.CONFIGS["tiny"]
    cfg = I.model_cfg(c)
    params = I.make_params(cfg, c["seed"])
    big = I.make_batch(c)                                        # 8 sentences x 10 tokens
    small = I.make_batch(c, batch=5, len_range=(3, 7), seed=11)  # ragged, fewer and shorter sentences
    tr = binding.Trainer(cfg, 8, 10, 10, precision=prec)
    try:
        tr.set_params(I.flatten(params, cfg))
        dev_big, dev_small = tr.upload_batch(*big), tr.upload_batch(*small)
        want_big, want_small = tr.eval_loss(dev_big), tr.eval_loss(dev_small)
        # a training step in between: its gradients and intermediates must survive the static calls
        loss_train = tr.train_step(dev_big)
        grads = tr.get_grads()
        h_o = tr.debug_fetch("h_o", (10, tr.padded_batch(), cfg["hidden"]))
        got_big = tr.eval_loss_static(dev_big)
        got_small = tr.eval_loss_static(dev_small)
        assert got_big == want_big, (got_big, want_big)
        assert got_small == want_small, (got_small, want_small)
        assert got_big[1] == float(big[3].sum()) and got_small[1] == float(small[3].sum())
        assert np.isfinite(got_big[0]) and abs(got_big[0] - np.log(1000.0)) < 0.1
        # the handle's own state is untouched
        assert np.array_equal(tr.get_grads(), grads)
        assert np.array_equal(tr.debug_fetch("h_o", h_o.shape), h_o)
        assert tr.train_step(dev_big) == loss_train
        # and once more after the step, larger input after the smaller one
        assert tr.eval_loss_static(dev_big) == want_big
    finally:
        tr.close()


def test_static_eval_matches_workspace_eval_fp32():
    _case(0)


def test_static_eval_matches_workspace_eval_bf16():
    _case(1)


def test_static_eval_refuses_a_shape_beyond_the_array():
    from paper_1802_07170_amd import binding
    c = I.CONFIGS["small"]                                       # vocabulary 32000: the slab buffers alone exceed the array
    cfg = I.model_cfg(c)
    batch = I.make_batch(c, batch=4, len_range=(5, 8), seed=3)
    tr = binding.Trainer(cfg, 4, 8, 8, precision=1)
    try:
        tr.init_params(1, 0.1)
        dev = tr.upload_batch(*batch)
        want = tr.eval_loss(dev)
        with pytest.raises(binding.CmtError) as e:
            tr.eval_loss_static(dev)
        assert e.value.code == binding.CMT_EINVAL and "static buffer holds" in str(e.value)
        assert tr.eval_loss(dev) == want                         # still usable
    finally:
        tr.close()
