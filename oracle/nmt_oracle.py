"""Plain fp64 CPU oracle of one training step of the attention-based stacked-LSTM
encoder-decoder (the paper's Method section, Eq. 1-7, with the hyperparameter table's
"bidirectional encoder" and "LSTM" choices).

THIS IS TEST INFRASTRUCTURE.  It is slow, written to be checked against the paper by eye, and
shares no code with the HIP library.  Only tests, the smoke check and the benchmark's CPU-baseline
leg may import it; the product path never does.

What it computes, per sentence pair (all sentences of a batch are independent):
  * embeddings are rows of E_src / E_tgt (the paper's EmbeddingLayer);
  * the encoder is a stack of LSTM layers; the bottom one is bidirectional (two LSTMs of width
    H/2 whose outputs are concatenated), the others run forward only;
  * the decoder is a stack of LSTM layers whose bottom layer input is [emb(y_{j-1}); H_o^{<j-1>}]
    (input feeding, H_o^{<-1>} = 0); decoder layer l starts from the encoder layer l final state;
  * attention, in the paper's order (Fig. "Attention", Eq. 3-7): q = W_a H_t, F_a[i] = H_s[i].q,
    a = softmax_i(F_a) over valid source positions, C_s = sum_i a_i H_s[i], C_st = [C_s; H_t],
    H_o = tanh(W_c C_st);
  * Eq. 1: z = W_o H_o + B_o, nll_j = logsumexp(z) - z[y_j]; loss = sum of nll / #target tokens.
    Eq. 1 as printed wraps the logits in an extra tanh; `logit_tanh=True` gives that literal
    reading (default off, see the design notes for why).
The backward pass is written by hand from these definitions: a weight used at every step sums its
per-step gradients (the paper's calculateGradient accumulates with beta = 1), and a value with two
consumers sums their gradients (the paper's DuplicateLayer).

greedy_decode and beam_decode are the forward-only companions (hyperparameter table: beam search
size 10, length penalty 0.6): the same encoder and decoder step, the arg-max token or the best
`beam` extensions fed back.

Regularisation of the Settings section / hyperparameter table (both off by default):
  * dropout p on the hidden states passed from a recurrent layer to the layer above it (encoder and
    decoder, every layer but the top one; the recurrent connection itself is not dropped) and on
    the output H_o: a kept entry is scaled by 1/(1-p); the dropped H_o is what the output layer and
    the next step's input feed see.  The masks come from a counter-based generator (dropout_mask);
  * label smoothing eps: the target distribution of Eq. 1 becomes (1-eps) onehot(y) + eps/V, so a
    token's loss is (1-eps) nll + eps (lse - mean_v z_v).

Readings of points the paper leaves open: gate order i, f, g, o in the packed weight rows, one
bias per gate, no peepholes, initial encoder state zero, no bias on W_a and W_c, padded source
positions get attention weight exactly 0, a padded step leaves the LSTM state unchanged and emits
a zero output.

Parity pins (tests/test_oracle_*.py): central finite differences on every parameter tensor,
closed-form LSTM outputs for zero / bias-only / saturated gates, torch.nn.LSTM (fp64) on random
inputs, torch.log_softmax, a torch-autograd restatement of the full model, padded-batch ==
per-sentence brute force, attention rows summing to one, loss == log V for a zero output layer;
dropout and label smoothing: finite differences with the masks held fixed, the same torch
restatement with masks and torch's own label-smoothed cross-entropy, SplitMix64's published first
outputs, keep rate and values of the masks; the optional operand-rounding model: identity hook ==
plain result bit for bit, bf16_round against hand-computed values, a one-step product against the
same product of hand-rounded inputs.  No function here is unpinned.
"""
from __future__ import annotations

import contextlib

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------------
# parameter table (canonical order, row-major [out, in])
# ----------------------------------------------------------------------------------------------
def param_shapes(cfg):
    """List of (name, shape).  cfg: dict with src_vocab, tgt_vocab, emb, hidden, layers."""
    Vs, Vt, E, H, L = cfg["src_vocab"], cfg["tgt_vocab"], cfg["emb"], cfg["hidden"], cfg["layers"]
    assert H % 2 == 0
    Hd = H // 2
    out = [("E_src", (Vs, E)), ("E_tgt", (Vt, E))]
    for d in ("fwd", "bwd"):
        out += [(f"enc.l0.{d}.W", (4 * Hd, E + Hd)), (f"enc.l0.{d}.b", (4 * Hd,))]
    for l in range(1, L):
        out += [(f"enc.l{l}.W", (4 * H, 2 * H)), (f"enc.l{l}.b", (4 * H,))]
    out += [("dec.l0.W", (4 * H, E + H + H)), ("dec.l0.b", (4 * H,))]
    for l in range(1, L):
        out += [(f"dec.l{l}.W", (4 * H, 2 * H)), (f"dec.l{l}.b", (4 * H,))]
    out += [("W_a", (H, H)), ("W_c", (H, 2 * H)), ("W_o", (Vt, H)), ("B_o", (Vt,))]
    return out


# ----------------------------------------------------------------------------------------------
# optional precision model (off by default: every contraction below is exact fp64)
# ----------------------------------------------------------------------------------------------
# The bf16 path of the library under test stores every matrix-product operand (weights, embeddings,
# LSTM states, attention keys, context, H_o, gate / logit gradients) as bfloat16 and accumulates in
# fp32.  `operand_rounding(fn)` turns this oracle into the matching precision model: while it is
# active, fn is applied to the matrix operands of every contraction (matrix product or attention
# einsum), forward and backward; the softmax coefficients and the fp32-resident gradient vectors
# (a, ds, dC_s), every sum and all pointwise arithmetic stay exact.  Tests use it with bf16_round to
# ask how far ANY bf16-operand method can be from the exact gradient on a given input (the
# conditioning of that gradient); nothing else uses it.
_operand_fn = None


def _op(x):
    return x if _operand_fn is None else _operand_fn(x)


@contextlib.contextmanager
def operand_rounding(fn):
    global _operand_fn
    prev, _operand_fn = _operand_fn, fn
    try:
        yield
    finally:
        _operand_fn = prev


def bf16_round(x):
    """Nearest bfloat16 value (ties to even) of every element, returned as float64."""
    x32 = np.ascontiguousarray(x, np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x32.shape).astype(F64)


def sigmoid(x):
    # identical to 1/(1+exp(-x)); this form cannot overflow
    return 0.5 * (1.0 + np.tanh(0.5 * x))


# ----------------------------------------------------------------------------------------------
# LSTM cell (hyperparameter table: "RNN type LSTM"): one step for a whole batch
# ----------------------------------------------------------------------------------------------
def cell_forward(x, h_prev, c_prev, W, b):
    """x [B,K], h_prev/c_prev [B,h], W [4h, K+h] (rows: i,f,g,o blocks; columns: [x; h]), b [4h]."""
    h = h_prev.shape[1]
    xh = np.concatenate([x, h_prev], axis=1)
    pre = _op(xh) @ _op(W).T + b
    i = sigmoid(pre[:, 0 * h:1 * h])
    f = sigmoid(pre[:, 1 * h:2 * h])
    g = np.tanh(pre[:, 2 * h:3 * h])
    o = sigmoid(pre[:, 3 * h:4 * h])
    c_new = f * c_prev + i * g
    h_new = o * np.tanh(c_new)
    cache = dict(xh=xh, i=i, f=f, g=g, o=o, c_prev=c_prev, c_new=c_new)
    return h_new, c_new, cache


def cell_backward(dh_new, dc_new, cache, W):
    """Gradients of one cell step.  Returns dx, dh_prev, dc_prev, dW, db."""
    i, f, g, o = cache["i"], cache["f"], cache["g"], cache["o"]
    c_prev, c_new, xh = cache["c_prev"], cache["c_new"], cache["xh"]
    h = i.shape[1]
    tc = np.tanh(c_new)
    do = dh_new * tc
    dc = dc_new + dh_new * o * (1.0 - tc * tc)
    di = dc * g
    df = dc * c_prev
    dg = dc * i
    dc_prev = dc * f
    dpre = np.concatenate([di * i * (1 - i), df * f * (1 - f), dg * (1 - g * g), do * o * (1 - o)], axis=1)
    dxh = _op(dpre) @ _op(W)
    K = xh.shape[1] - h
    dW = _op(dpre).T @ _op(xh)
    db = dpre.sum(axis=0)
    return dxh[:, :K], dxh[:, K:], dc_prev, dW, db


def masked_step_forward(x, h_prev, c_prev, m, W, b):
    """One step with a 0/1 mask column m [B,1]: a masked row keeps its state and emits y = 0."""
    h_new, c_new, cache = cell_forward(x, h_prev, c_prev, W, b)
    h = m * h_new + (1 - m) * h_prev
    c = m * c_new + (1 - m) * c_prev
    y = m * h_new
    cache["m"] = m
    return y, h, c, cache


def masked_step_backward(dy, dh_state, dc_state, cache, W):
    """dy: gradient of the emitted y; dh_state/dc_state: gradient of the state after the step."""
    m = cache["m"]
    dh_new = m * (dh_state + dy)
    dc_new = m * dc_state
    dx, dh_prev, dc_prev, dW, db = cell_backward(dh_new, dc_new, cache, W)
    dh_prev = dh_prev + (1 - m) * dh_state
    dc_prev = dc_prev + (1 - m) * dc_state
    return dx, dh_prev, dc_prev, dW, db


def lstm_forward(X, mask, W, b, h0, c0, reverse=False):
    """A whole LSTM layer (one direction) over X [T,B,K] with mask [T,B].
    Returns Y [T,B,h] (zero on masked steps), final (h, c), and the per-step caches."""
    T = X.shape[0]
    order = range(T - 1, -1, -1) if reverse else range(T)
    h, c = h0, c0
    Y = np.zeros((T,) + h0.shape, F64)
    Hst = np.zeros_like(Y)
    Cst = np.zeros_like(Y)
    caches = [None] * T
    for t in order:
        Y[t], h, c, caches[t] = masked_step_forward(X[t], h, c, mask[t][:, None], W, b)
        Hst[t], Cst[t] = h, c
    return Y, h, c, dict(caches=caches, reverse=reverse, Hst=Hst, Cst=Cst)


def lstm_backward(dY, dh_final, dc_final, saved, W):
    """Backward of lstm_forward.  Returns dX, dW, db, dh0, dc0."""
    caches, reverse = saved["caches"], saved["reverse"]
    T = len(caches)
    order = range(T) if reverse else range(T - 1, -1, -1)   # reverse of the processing order
    dh, dc = dh_final, dc_final
    dW = np.zeros_like(W)
    db = np.zeros(W.shape[0], F64)
    dX = None
    for t in order:
        dx, dh, dc, dWt, dbt = masked_step_backward(dY[t], dh, dc, caches[t], W)
        if dX is None:
            dX = np.zeros((T,) + dx.shape, F64)
        dX[t] = dx
        dW += dWt
        db += dbt
    return dX, dW, db, dh, dc


# ----------------------------------------------------------------------------------------------
# attention (Eq. 3-7) for one decoder step, whole batch
# ----------------------------------------------------------------------------------------------
def attention_forward(Hs, src_mask, Ht, W_a, W_c):
    """Hs [S,B,H], src_mask [S,B] (1 = valid), Ht [B,H].  Returns H_o [B,H] and a cache."""
    q = _op(Ht) @ _op(W_a).T                                   # W_a H_t  (linearHt in the paper's listing)
    s = np.einsum("ibh,bh->bi", _op(Hs), _op(q))               # F_a = H_s^T (W_a H_t), Eq. 4
    valid = src_mask.T > 0                           # [B,S]
    s = np.where(valid, s, -np.inf)
    smax = s.max(axis=1, keepdims=True)
    e = np.where(valid, np.exp(s - smax), 0.0)
    a = e / e.sum(axis=1, keepdims=True)             # Eq. 3
    Cs = np.einsum("bi,ibh->bh", a, _op(Hs))              # Eq. 5
    Cst = np.concatenate([Cs, Ht], axis=1)           # Eq. 6
    Ho = np.tanh(_op(Cst) @ _op(W_c).T)                        # Eq. 7
    return Ho, dict(q=q, s=s, a=a, Cs=Cs, Cst=Cst, Ho=Ho, Ht=Ht)


def attention_backward(dHo, cache, Hs, W_a, W_c):
    """Returns dHt [B,H], dHs [S,B,H], dW_a, dW_c."""
    a, q, Cst, Ho, Ht = cache["a"], cache["q"], cache["Cst"], cache["Ho"], cache["Ht"]
    H = Ht.shape[1]
    dpre = dHo * (1.0 - Ho * Ho)
    dW_c = _op(dpre).T @ _op(Cst)
    dCst = _op(dpre) @ _op(W_c)
    dCs, dHt = dCst[:, :H], dCst[:, H:].copy()       # the second consumer of H_t (DuplicateLayer)
    da = np.einsum("ibh,bh->bi", _op(Hs), dCs)
    dHs = np.einsum("bi,bh->ibh", a, dCs)
    ds = a * (da - (a * da).sum(axis=1, keepdims=True))
    dq = np.einsum("bi,ibh->bh", ds, _op(Hs))
    dHs += np.einsum("bi,bh->ibh", ds, q)
    dW_a = _op(dq).T @ _op(Ht)
    dHt += _op(dq) @ _op(W_a)
    return dHt, dHs, dW_a, dW_c


# ----------------------------------------------------------------------------------------------
# output layer (Eq. 1) for one decoder step, whole batch
# ----------------------------------------------------------------------------------------------
def output_forward(Ho, labels, W_o, B_o, logit_tanh=False, label_smoothing=0.0):
    """Returns lse [B], the per-row loss [B] (unmasked), cache.  The row loss is the cross-entropy
    against the target distribution q = (1 - eps) onehot(label) + eps / V (eps = 0: plain nll)."""
    u = _op(Ho) @ _op(W_o).T + B_o
    z = np.tanh(u) if logit_tanh else u
    zmax = z.max(axis=1, keepdims=True)
    lse = (zmax + np.log(np.exp(z - zmax).sum(axis=1, keepdims=True)))[:, 0]
    nll = lse - z[np.arange(z.shape[0]), labels]
    eps = label_smoothing
    row = (1.0 - eps) * nll + eps * (lse - z.mean(axis=1))      # -sum_v q_v log p_v
    return lse, row, dict(z=z, lse=lse, labels=labels, Ho=Ho, logit_tanh=logit_tanh, eps=eps)


def output_backward(w, cache, W_o):
    """w [B]: d loss / d (row loss) per row (mask / N_tok).  Returns dHo, dW_o, dB_o."""
    z, lse, labels, Ho = cache["z"], cache["lse"], cache["labels"], cache["Ho"]
    eps = cache["eps"]
    dz = np.exp(z - lse[:, None])                                # p - q
    dz[np.arange(z.shape[0]), labels] -= 1.0 - eps
    dz -= eps / z.shape[1]
    dz *= w[:, None]
    if cache["logit_tanh"]:
        dz = dz * (1.0 - z * z)
    return _op(dz) @ _op(W_o), _op(dz).T @ _op(Ho), dz.sum(axis=0)


# ----------------------------------------------------------------------------------------------
# the whole training step
# ----------------------------------------------------------------------------------------------
def make_masks(src_len, tgt_len, S, T):
    src_mask = (np.arange(S)[:, None] < np.asarray(src_len)[None, :]).astype(F64)   # [S,B]
    tgt_mask = (np.arange(T)[:, None] < np.asarray(tgt_len)[None, :]).astype(F64)   # [T,B]
    return src_mask, tgt_mask


def splitmix64(x):
    """The SplitMix64 output function on uint64 arrays: x + golden gamma, then the two
    xor-shift-multiply rounds and the final xor-shift (the published generator's step)."""
    with np.errstate(over="ignore"):
        x = x + np.uint64(0x9E3779B97F4A7C15)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return x ^ (x >> np.uint64(31))


DROPOUT_SITE_ENC, DROPOUT_SITE_DEC, DROPOUT_SITE_HO = 0, 16, 32   # + layer number for the first two


def dropout_mask(seed, site, T, B, H, p):
    """Keep-and-rescale factors [T,B,H] of one dropout site.  Element (t, b, h) is kept iff the top
    24 bits of SplitMix64(seed + site * 2^48 + (t B + b) H + h) are >= floor(float32(p) * 2^24);
    kept entries are 1 / (1 - p), dropped ones 0.  B is the real batch size, so the masks do not
    depend on how a batch is padded."""
    if p <= 0.0:
        return np.ones((T, B, H), F64)
    n = T * B * H
    key = (np.arange(n, dtype=np.uint64) + np.uint64((int(seed) + (int(site) << 48)) & ((1 << 64) - 1)))
    u = (splitmix64(key) >> np.uint64(40)).astype(np.int64)
    thresh = int(np.floor(float(np.float32(p)) * 16777216.0))
    return ((u >= thresh).astype(F64) / (1.0 - float(np.float32(p)))).reshape(T, B, H)


def train_step(cfg, params, src_ids, src_len, tgt_ids, tgt_len, bos_id=2, logit_tanh=False,
               want_intermediates=False, dropout=0.0, dropout_seed=0, label_smoothing=0.0):
    """One forward + backward pass.

    params: dict name -> float64 array (see param_shapes).  src_ids [B,S], tgt_ids [B,T] int;
    src_len, tgt_len [B] with 1 <= len <= S (T).  Decoder input at step j is BOS for j = 0, else
    tgt_ids[:, j-1]; the label at step j is tgt_ids[:, j].
    Returns (loss, grads dict, intermediates dict or None)."""
    p = {k: np.asarray(v, F64) for k, v in params.items()}
    src_ids = np.asarray(src_ids)
    tgt_ids = np.asarray(tgt_ids)
    B, S = src_ids.shape
    T = tgt_ids.shape[1]
    H, L = cfg["hidden"], cfg["layers"]
    Hd = H // 2
    src_mask, tgt_mask = make_masks(src_len, tgt_len, S, T)
    n_tok = float(np.sum(tgt_len))

    # ---- embeddings -------------------------------------------------------------------------
    dec_in = np.concatenate([np.full((B, 1), bos_id, tgt_ids.dtype), tgt_ids[:, :T - 1]], axis=1)
    Xs = p["E_src"][src_ids.T]                      # [S,B,E]
    Xt = p["E_tgt"][dec_in.T]                       # [T,B,E]

    # ---- encoder ----------------------------------------------------------------------------
    z_d = np.zeros((B, Hd), F64)
    z_h = np.zeros((B, H), F64)
    Yf, hf, cf, sv_f = lstm_forward(Xs, src_mask, p["enc.l0.fwd.W"], p["enc.l0.fwd.b"], z_d, z_d)
    Yb, hb, cb, sv_b = lstm_forward(Xs, src_mask, p["enc.l0.bwd.W"], p["enc.l0.bwd.b"], z_d, z_d, reverse=True)
    enc_Y = [np.concatenate([Yf, Yb], axis=2)]
    enc_fin = [(np.concatenate([hf, hb], axis=1), np.concatenate([cf, cb], axis=1))]
    enc_sv = [(sv_f, sv_b)]
    D_enc = [dropout_mask(dropout_seed, DROPOUT_SITE_ENC + l, S, B, H, dropout) for l in range(L - 1)]
    D_dec = [dropout_mask(dropout_seed, DROPOUT_SITE_DEC + l, T, B, H, dropout) for l in range(L - 1)]
    D_ho = dropout_mask(dropout_seed, DROPOUT_SITE_HO, T, B, H, dropout)
    for l in range(1, L):
        Y, h, c, sv = lstm_forward(enc_Y[-1] * D_enc[l - 1], src_mask, p[f"enc.l{l}.W"], p[f"enc.l{l}.b"], z_h, z_h)
        enc_Y.append(Y)
        enc_fin.append((h, c))
        enc_sv.append(sv)
    Hs = enc_Y[-1]                                   # source-side top-layer states

    # ---- decoder, attention and output, step by step -----------------------------------------
    h = [enc_fin[l][0] for l in range(L)]
    c = [enc_fin[l][1] for l in range(L)]
    Ho_prev = z_h
    dec_caches, att_caches, out_caches, dec_states = [], [], [], []
    nll_all = np.zeros((T, B), F64)
    lse_all = np.zeros((T, B), F64)
    for j in range(T):
        m = tgt_mask[j][:, None]
        x = np.concatenate([Xt[j], Ho_prev], axis=1)
        step_caches = []
        for l in range(L):
            _, h[l], c[l], cache = masked_step_forward(x, h[l], c[l], m, p[f"dec.l{l}.W"], p[f"dec.l{l}.b"])
            step_caches.append(cache)
            x = h[l] * D_dec[l][j] if l < L - 1 else h[l]
        Ho, acache = attention_forward(Hs, src_mask, h[L - 1], p["W_a"], p["W_c"])
        Ho_d = Ho * D_ho[j]                          # what the output layer and the input feed see
        lse, nll, ocache = output_forward(Ho_d, tgt_ids[:, j], p["W_o"], p["B_o"], logit_tanh, label_smoothing)
        nll_all[j], lse_all[j] = nll, lse
        dec_caches.append(step_caches)
        dec_states.append(([hl.copy() for hl in h], [cl.copy() for cl in c]))
        att_caches.append(acache)
        out_caches.append(ocache)
        Ho_prev = Ho_d
    loss = float((nll_all * tgt_mask).sum() / n_tok)

    # ---- backward ---------------------------------------------------------------------------
    g = {k: np.zeros_like(v) for k, v in p.items()}
    dHs = np.zeros_like(Hs)
    dh = [np.zeros((B, H), F64) for _ in range(L)]
    dc = [np.zeros((B, H), F64) for _ in range(L)]
    dHo_feed = np.zeros((B, H), F64)
    dXt = np.zeros_like(Xt)
    E = Xt.shape[2]
    for j in range(T - 1, -1, -1):
        dHo, dWo, dBo = output_backward(tgt_mask[j] / n_tok, out_caches[j], p["W_o"])
        g["W_o"] += dWo
        g["B_o"] += dBo
        dHo = (dHo + dHo_feed) * D_ho[j]
        dHt, dHs_j, dWa, dWc = attention_backward(dHo, att_caches[j], Hs, p["W_a"], p["W_c"])
        g["W_a"] += dWa
        g["W_c"] += dWc
        dHs += dHs_j
        dy = dHt                                     # gradient reaching the top layer's output
        for l in range(L - 1, -1, -1):
            dx, dh[l], dc[l], dW, db = masked_step_backward(
                np.zeros_like(dy), dh[l] + dy, dc[l], dec_caches[j][l], p[f"dec.l{l}.W"])
            g[f"dec.l{l}.W"] += dW
            g[f"dec.l{l}.b"] += db
            dy = dx * D_dec[l - 1][j] if l > 0 else dx
        dXt[j] = dy[:, :E]
        dHo_feed = dy[:, E:]
    # (H_o^{<-1>} is the constant zero vector: the last dHo_feed is dropped.)

    # decoder initial states are the encoder final states
    dHs *= src_mask[:, :, None]                      # H_s at padded positions is the constant 0
    dY = dHs
    for l in range(L - 1, 0, -1):
        dY, dW, db, _, _ = lstm_backward(dY, dh[l], dc[l], enc_sv[l], p[f"enc.l{l}.W"])
        dY = dY * D_enc[l - 1]
        g[f"enc.l{l}.W"] += dW
        g[f"enc.l{l}.b"] += db
    sv_f, sv_b = enc_sv[0]
    dXf, dW, db, _, _ = lstm_backward(dY[:, :, :Hd], dh[0][:, :Hd], dc[0][:, :Hd], sv_f, p["enc.l0.fwd.W"])
    g["enc.l0.fwd.W"] += dW
    g["enc.l0.fwd.b"] += db
    dXb, dW, db, _, _ = lstm_backward(dY[:, :, Hd:], dh[0][:, Hd:], dc[0][:, Hd:], sv_b, p["enc.l0.bwd.W"])
    g["enc.l0.bwd.W"] += dW
    g["enc.l0.bwd.b"] += db
    dXs = dXf + dXb

    # embedding rows: every occurrence adds its gradient (padded slots carry exactly zero)
    np.add.at(g["E_src"], src_ids.T.reshape(-1), dXs.reshape(-1, dXs.shape[2]))
    np.add.at(g["E_tgt"], dec_in.T.reshape(-1), dXt.reshape(-1, E))

    inter = None
    if want_intermediates:
        inter = dict(
            x_src=Xs, x_tgt=Xt, mask_src=src_mask, mask_tgt=tgt_mask, h_s=Hs,
            att_a=np.stack([ac["a"] for ac in att_caches]),          # [T,B,S]
            att_cs=np.stack([ac["Cs"] for ac in att_caches]),        # [T,B,H]
            h_t=np.stack([ac["Ht"] for ac in att_caches]),           # [T,B,H]
            h_o=np.stack([ac["Ho"] for ac in att_caches]),           # [T,B,H], before dropout
            h_o_drop=np.stack([ac["Ho"] for ac in att_caches]) * D_ho,
            lse=lse_all, nll=nll_all * tgt_mask,
            enc_y=enc_Y, enc_final=enc_fin,
            att_s=np.stack([ac["s"] for ac in att_caches]),          # [T,B,S] scores of Eq. 4, -inf on padding
        )
        # per LSTM (layer, direction): state after every step (h, c) and the gate activations [i, f, g, o]
        gates = lambda caches: np.stack([np.concatenate([ch["i"], ch["f"], ch["g"], ch["o"]], axis=1) for ch in caches])
        for name, sv in [("enc.l0.fwd", enc_sv[0][0]), ("enc.l0.bwd", enc_sv[0][1])] + [(f"enc.l{l}", enc_sv[l]) for l in range(1, L)]:
            inter[name + ".h"], inter[name + ".c"], inter[name + ".gates"] = sv["Hst"], sv["Cst"], gates(sv["caches"])
        for l in range(L):
            inter[f"dec.l{l}.h"] = np.stack([st[0][l] for st in dec_states])
            inter[f"dec.l{l}.c"] = np.stack([st[1][l] for st in dec_states])
            inter[f"dec.l{l}.gates"] = gates([dec_caches[j][l] for j in range(T)])
    return loss, g, inter


def greedy_decode(cfg, params, src_ids, src_len, max_len, bos_id=2, eos_id=3, pad_id=0):
    """Forward-only translation with the arg-max token fed back (beam size 1; no dropout).

    The encoder and one decoder step are exactly those of train_step.  At step j the decoder input is
    BOS (j = 0) or the previous output token; the output token is argmax_v (W_o H_o + B_o)_v, the
    lowest index winning a tie.  A sentence ends with the step that emits eos_id (kept in the output)
    or at step max_len - 1.  Returns ids [B, max_len] (pad_id after the end), lengths [B], and for
    every emitted token the gap between the best and second-best logit [B, max_len] (inf after the
    end), which tells a parity test how close to a tie a decision was."""
    p = {k: np.asarray(v, F64) for k, v in params.items()}
    src_ids = np.asarray(src_ids)
    B, S = src_ids.shape
    H, L = cfg["hidden"], cfg["layers"]
    Hd = H // 2
    src_mask, _ = make_masks(src_len, np.ones(B, int), S, 1)
    Xs = p["E_src"][src_ids.T]
    z_d = np.zeros((B, Hd), F64)
    z_h = np.zeros((B, H), F64)
    Yf, hf, cf, _ = lstm_forward(Xs, src_mask, p["enc.l0.fwd.W"], p["enc.l0.fwd.b"], z_d, z_d)
    Yb, hb, cb, _ = lstm_forward(Xs, src_mask, p["enc.l0.bwd.W"], p["enc.l0.bwd.b"], z_d, z_d, reverse=True)
    Y = np.concatenate([Yf, Yb], axis=2)
    h = [np.concatenate([hf, hb], axis=1)]
    c = [np.concatenate([cf, cb], axis=1)]
    for l in range(1, L):
        Y, hl, cl, _ = lstm_forward(Y, src_mask, p[f"enc.l{l}.W"], p[f"enc.l{l}.b"], z_h, z_h)
        h.append(hl)
        c.append(cl)
    Hs = Y
    ids = np.full((B, max_len), pad_id, np.int64)
    lens = np.zeros(B, np.int64)
    gaps = np.full((B, max_len), np.inf)
    done = np.zeros(B, bool)
    tok = np.full(B, bos_id, np.int64)
    Ho = z_h
    ones = np.ones((B, 1), F64)
    for j in range(max_len):
        x = np.concatenate([p["E_tgt"][tok], Ho], axis=1)
        for l in range(L):
            _, h[l], c[l], _ = masked_step_forward(x, h[l], c[l], ones, p[f"dec.l{l}.W"], p[f"dec.l{l}.b"])
            x = h[l]
        Ho, _ = attention_forward(Hs, src_mask, h[L - 1], p["W_a"], p["W_c"])
        z = Ho @ p["W_o"].T + p["B_o"]
        tok = z.argmax(axis=1)                       # first maximum = lowest index
        top2 = np.partition(z, -2, axis=1)[:, -2:]
        for b in range(B):
            if done[b]:
                continue
            ids[b, j] = tok[b]
            gaps[b, j] = top2[b, 1] - top2[b, 0]
            if tok[b] == eos_id or j == max_len - 1:
                done[b] = True
                lens[b] = j + 1
    return ids, lens, gaps


def length_penalty(length, alpha):
    """Length normalisation of Wu et al. (2016), which the paper's Settings section names:
    lp(Y) = ((5 + |Y|) / 6) ** alpha."""
    return ((5.0 + length) / 6.0) ** alpha


def beam_decode(cfg, params, src_ids, src_len, max_len, beam, alpha, bos_id=2, eos_id=3, pad_id=0):
    """Beam search (hyperparameter table: beam size 10, length penalty 0.6), sentence by sentence.

    A hypothesis carries the sum of log p(token) of its tokens.  At every step the `beam` best
    one-token extensions over all live hypotheses are taken (equal scores: the lower (hypothesis
    slot, token) pair first).  An extension that ends in eos_id leaves the beam as a finished
    hypothesis of length = its number of tokens (eos included); the others stay live, best first.
    A sentence is done when no hypothesis is live or after max_len steps; hypotheses still live then
    are finished as they are.  The result is the finished hypothesis with the largest
    score / length_penalty(length, alpha) (equal values: the one finished first).  No dropout.

    Returns ids [B, max_len] (pad_id after the end), lengths [B], normalised scores [B], and
    margins [B]: the smallest score gap met at any decision that shaped the result (the beam
    boundary at every step, and the final winner against the runner-up), for parity tests."""
    p = {k: np.asarray(v, F64) for k, v in params.items()}
    src_ids = np.asarray(src_ids)
    B = src_ids.shape[0]
    H, L = cfg["hidden"], cfg["layers"]
    Hd = H // 2
    out_ids = np.full((B, max_len), pad_id, np.int64)
    out_len = np.zeros(B, np.int64)
    out_score = np.zeros(B, F64)
    margins = np.full(B, np.inf)
    for b in range(B):
        n = int(src_len[b])
        Xs = p["E_src"][src_ids[b, :n]][:, None, :]              # [n, 1, E]
        m1 = np.ones((n, 1), F64)
        z_d, z_h = np.zeros((1, Hd), F64), np.zeros((1, H), F64)
        Yf, hf, cf, _ = lstm_forward(Xs, m1, p["enc.l0.fwd.W"], p["enc.l0.fwd.b"], z_d, z_d)
        Yb, hb, cb, _ = lstm_forward(Xs, m1, p["enc.l0.bwd.W"], p["enc.l0.bwd.b"], z_d, z_d, reverse=True)
        Y = np.concatenate([Yf, Yb], axis=2)
        h = [np.concatenate([hf, hb], axis=1)]
        c = [np.concatenate([cf, cb], axis=1)]
        for l in range(1, L):
            Y, hl, cl, _ = lstm_forward(Y, m1, p[f"enc.l{l}.W"], p[f"enc.l{l}.b"], z_h, z_h)
            h.append(hl)
            c.append(cl)
        Hs1 = Y                                                   # [n, 1, H]
        live_tok = [[]]                                           # token lists of the live hypotheses
        live_score = np.zeros(1, F64)
        prev = np.array([bos_id])
        Ho = z_h
        finished = []                                             # (normalised score, order, tokens)
        for j in range(max_len):
            k = len(live_tok)
            x = np.concatenate([p["E_tgt"][prev], Ho], axis=1)
            ones = np.ones((k, 1), F64)
            for l in range(L):
                _, h[l], c[l], _ = masked_step_forward(x, h[l], c[l], ones, p[f"dec.l{l}.W"], p[f"dec.l{l}.b"])
                x = h[l]
            Hs = np.repeat(Hs1, k, axis=1)
            Ho, _ = attention_forward(Hs, np.ones((n, k), F64), h[L - 1], p["W_a"], p["W_c"])
            z = Ho @ p["W_o"].T + p["B_o"]
            zmax = z.max(axis=1, keepdims=True)
            logp = z - (zmax + np.log(np.exp(z - zmax).sum(axis=1, keepdims=True)))
            cand = (live_score[:, None] + logp).reshape(-1)       # flat index = slot * V + token
            order = np.lexsort((np.arange(cand.size), -cand))     # by score descending, then flat index
            top = order[:beam]
            if cand.size > beam:
                margins[b] = min(margins[b], cand[order[beam - 1]] - cand[order[beam]])
            V = z.shape[1]
            new_tok, new_score, parents = [], [], []
            for rank, f in enumerate(top):
                slot, tok = int(f // V), int(f % V)
                seq = live_tok[slot] + [tok]
                if tok == eos_id or j == max_len - 1:
                    finished.append((cand[f] / length_penalty(len(seq), alpha), len(finished), seq))
                else:
                    new_tok.append(seq)
                    new_score.append(cand[f])
                    parents.append(slot)
            if not new_tok:
                break
            live_tok, live_score = new_tok, np.array(new_score)
            h = [hh[parents] for hh in h]
            c = [cc[parents] for cc in c]
            Ho = Ho[parents]
            prev = np.array([seq[-1] for seq in live_tok])
        finished.sort(key=lambda t: (-t[0], t[1]))
        best = finished[0]
        if len(finished) > 1:
            margins[b] = min(margins[b], best[0] - finished[1][0])
        out_ids[b, :len(best[2])] = best[2]
        out_len[b] = len(best[2])
        out_score[b] = best[0]
    return out_ids, out_len, out_score, margins


def sgd_update(params, grads, lr):
    """Plain SGD (hyperparameter table: optimizer SGD): p <- p - lr * g."""
    return {k: np.asarray(params[k], F64) - lr * grads[k] for k in params}


def init_params_counter(cfg, seed, scale):
    """uniform[-scale, scale) parameters from a counter-based generator: element number n of the
    flat canonical parameter vector is SplitMix64(seed + n)'s top 24 bits u, value
    (2 u / 2^24 - 1) * scale evaluated in float32.  The HIP library implements the same recipe
    independently, so results are bit-identical."""
    out = {}
    n0 = 0
    mask = (1 << 64) - 1
    for name, shape in param_shapes(cfg):
        n = int(np.prod(shape))
        idx = (np.arange(n0, n0 + n, dtype=np.uint64) + np.uint64(seed & mask))
        u = (splitmix64(idx) >> np.uint64(40)).astype(np.float32)  # 24 bits, exact in float32
        v = (u * np.float32(2.0 / 16777216.0) - np.float32(1.0)) * np.float32(scale)
        out[name] = v.astype(np.float32).reshape(shape)
        n0 += n
    return out
