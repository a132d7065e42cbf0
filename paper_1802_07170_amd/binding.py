"""Thin ctypes binding over the C ABI in include/cytonmt_hip.h: argument marshalling only.
torch is used for device memory and the stream; every step of the path runs in the HIP library.
There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcytonmt_hip.so")

CMT_OK, CMT_EINVAL, CMT_ERANGE, CMT_ENONFINITE, CMT_EHIP = 0, -1, -2, -3, -4

EXPORTS = [
    "cmt_query_sizes", "cmt_create", "cmt_destroy", "cmt_param_count", "cmt_param_info",
    "cmt_init_params", "cmt_set_params", "cmt_get_params", "cmt_train_step", "cmt_train_step_async",
    "cmt_fetch_loss", "cmt_get_grads", "cmt_sgd_update", "cmt_debug_fetch", "cmt_padded_batch",
    "cmt_time_kernel", "cmt_last_error", "cmt_set_regularization", "cmt_greedy_decode", "cmt_beam_decode",
    "cmt_eval_loss", "cmt_eval_loss_static",
]


class CmtConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "src_vocab", "tgt_vocab", "emb_dim", "hidden", "layers", "max_batch", "max_src_len",
        "max_tgt_len", "precision", "bos_id", "pad_id")]


class CmtError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"cytonmt_hip error {code}: {msg}")
        self.code = code


_lib = None


def load_library():
    """Loads the in-tree shared library (built by paper_1802_07170_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1802_07170_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    cfgp = C.POINTER(CmtConfig)
    lib.cmt_query_sizes.argtypes = [cfgp, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    lib.cmt_create.argtypes = [cfgp, vp, vp, vp, vp, C.POINTER(vp)]
    lib.cmt_destroy.argtypes = [vp]
    lib.cmt_destroy.restype = None
    lib.cmt_param_count.argtypes = [vp]
    lib.cmt_param_info.argtypes = [vp, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                   C.POINTER(C.c_int64), C.POINTER(sz)]
    lib.cmt_init_params.argtypes = [vp, C.c_uint64, C.c_float]
    lib.cmt_set_params.argtypes = [vp, vp]
    lib.cmt_get_params.argtypes = [vp, vp]
    lib.cmt_train_step.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, C.POINTER(C.c_float)]
    lib.cmt_train_step_async.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32]
    lib.cmt_fetch_loss.argtypes = [vp, C.POINTER(C.c_float)]
    lib.cmt_eval_loss.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.cmt_eval_loss_static.argtypes = lib.cmt_eval_loss.argtypes
    lib.cmt_get_grads.argtypes = [vp, vp]
    lib.cmt_sgd_update.argtypes = [vp, C.c_float]
    lib.cmt_set_regularization.argtypes = [vp, C.c_float, C.c_float, C.c_uint64]
    lib.cmt_greedy_decode.argtypes = [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp]
    lib.cmt_beam_decode.argtypes = [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_int32, vp, vp, vp]
    lib.cmt_debug_fetch.argtypes = [vp, C.c_char_p, vp, sz]
    lib.cmt_padded_batch.argtypes = [vp]
    lib.cmt_time_kernel.argtypes = [vp, C.c_char_p, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_double)]
    lib.cmt_last_error.argtypes = [vp]
    lib.cmt_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("cmt_destroy", "cmt_last_error"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def make_config(cfg, max_batch, max_src_len, max_tgt_len, precision, bos_id=2, pad_id=0):
    return CmtConfig(cfg["src_vocab"], cfg["tgt_vocab"], cfg["emb"], cfg["hidden"], cfg["layers"],
                     max_batch, max_src_len, max_tgt_len, precision, bos_id, pad_id)


def query_sizes(ccfg):
    lib = load_library()
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    rc = lib.cmt_query_sizes(C.byref(ccfg), C.byref(a), C.byref(b), C.byref(c))
    if rc != CMT_OK:
        raise CmtError(rc, "unsupported configuration")
    return a.value, b.value, c.value


class Trainer:
    """Owns the device buffers (torch tensors) and a library handle bound to them."""

    def __init__(self, cfg, max_batch, max_src_len, max_tgt_len, precision, bos_id=2, pad_id=0, device="cuda:0"):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.cfg = dict(cfg)
        self.ccfg = make_config(cfg, max_batch, max_src_len, max_tgt_len, precision, bos_id, pad_id)
        pb, gb, wb = query_sizes(self.ccfg)
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.n_params = pb // 4
        self.params = torch.empty(self.n_params, dtype=torch.float32, device=self.device)
        self.grads = torch.zeros(self.n_params, dtype=torch.float32, device=self.device)
        self.workspace = torch.zeros(wb, dtype=torch.uint8, device=self.device)
        self.workspace_bytes = wb
        self.stream = torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        rc = self.lib.cmt_create(C.byref(self.ccfg), self.params.data_ptr(), self.grads.data_ptr(),
                                 self.workspace.data_ptr(), self.stream.cuda_stream, C.byref(h))
        if rc != CMT_OK:
            raise CmtError(rc, "cmt_create failed")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.torch.cuda.synchronize(self.device)
            self.lib.cmt_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != CMT_OK:
            raise CmtError(rc, self.lib.cmt_last_error(self.h).decode())

    def param_table(self):
        out = []
        for i in range(self.lib.cmt_param_count(self.h)):
            name, r, c, off = C.c_char_p(), C.c_int64(), C.c_int64(), C.c_size_t()
            self._check(self.lib.cmt_param_info(self.h, i, C.byref(name), C.byref(r), C.byref(c), C.byref(off)))
            out.append((name.value.decode(), r.value, c.value, off.value))
        return out

    def init_params(self, seed, scale):
        self._check(self.lib.cmt_init_params(self.h, seed, scale))

    def set_params(self, flat):
        flat = np.ascontiguousarray(flat, dtype=np.float32)
        assert flat.size == self.n_params
        self._check(self.lib.cmt_set_params(self.h, flat.ctypes.data))

    def get_params(self):
        out = np.empty(self.n_params, np.float32)
        self._check(self.lib.cmt_get_params(self.h, out.ctypes.data))
        return out

    def get_grads(self):
        out = np.empty(self.n_params, np.float32)
        self._check(self.lib.cmt_get_grads(self.h, out.ctypes.data))
        return out

    def upload_batch(self, src_ids, src_len, tgt_ids, tgt_len):
        t = self.torch
        mk = lambda a: t.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.device)
        return mk(src_ids), mk(src_len), mk(tgt_ids), mk(tgt_len)

    def train_step(self, dev_batch):
        s, sl, tg, tl = dev_batch
        loss = C.c_float()
        self._check(self.lib.cmt_train_step(self.h, s.data_ptr(), sl.data_ptr(), tg.data_ptr(), tl.data_ptr(),
                                            s.shape[0], s.shape[1], tg.shape[1], C.byref(loss)))
        return loss.value

    def train_step_async(self, dev_batch):
        s, sl, tg, tl = dev_batch
        self._check(self.lib.cmt_train_step_async(self.h, s.data_ptr(), sl.data_ptr(), tg.data_ptr(), tl.data_ptr(),
                                                  s.shape[0], s.shape[1], tg.shape[1]))

    def fetch_loss(self):
        loss = C.c_float()
        self._check(self.lib.cmt_fetch_loss(self.h, C.byref(loss)))
        return loss.value

    def eval_loss(self, dev_batch):
        """Forward only, evaluation mode: (mean cross-entropy per valid target token, number of such tokens)."""
        s, sl, tg, tl = dev_batch
        loss, ntok = C.c_float(), C.c_float()
        self._check(self.lib.cmt_eval_loss(self.h, s.data_ptr(), sl.data_ptr(), tg.data_ptr(), tl.data_ptr(),
                                           s.shape[0], s.shape[1], tg.shape[1], C.byref(loss), C.byref(ntok)))
        return loss.value, ntok.value

    def eval_loss_static(self, dev_batch):
        """eval_loss with every intermediate in the library's static device array (allocates nothing)."""
        s, sl, tg, tl = dev_batch
        loss, ntok = C.c_float(), C.c_float()
        self._check(self.lib.cmt_eval_loss_static(self.h, s.data_ptr(), sl.data_ptr(), tg.data_ptr(), tl.data_ptr(),
                                                  s.shape[0], s.shape[1], tg.shape[1], C.byref(loss), C.byref(ntok)))
        return loss.value, ntok.value

    def sgd_update(self, lr):
        self._check(self.lib.cmt_sgd_update(self.h, lr))

    def greedy_decode(self, src_ids, src_len, max_len, eos_id=3):
        """Greedy translation of a batch (numpy int arrays in, numpy int32 arrays out): ids [B, max_len], lengths [B]."""
        torch = self.torch
        src = torch.from_numpy(np.ascontiguousarray(src_ids, np.int32)).to(self.device)
        sl = torch.from_numpy(np.ascontiguousarray(src_len, np.int32)).to(self.device)
        B, S = src.shape
        out = torch.empty((B, max_len), dtype=torch.int32, device=self.device)
        olen = torch.empty((B,), dtype=torch.int32, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.cmt_greedy_decode(self.h, src.data_ptr(), sl.data_ptr(), B, S, max_len, eos_id, out.data_ptr(),
                                               olen.data_ptr()))
        return out.cpu().numpy(), olen.cpu().numpy()

    def beam_decode(self, src_ids, src_len, max_len, beam=10, length_penalty=0.6, eos_id=3):
        """Beam search over a batch: ids [B, max_len], lengths [B], normalised scores [B] (numpy)."""
        torch = self.torch
        src = torch.from_numpy(np.ascontiguousarray(src_ids, np.int32)).to(self.device)
        sl = torch.from_numpy(np.ascontiguousarray(src_len, np.int32)).to(self.device)
        B, S = src.shape
        out = torch.empty((B, max_len), dtype=torch.int32, device=self.device)
        olen = torch.empty((B,), dtype=torch.int32, device=self.device)
        osc = torch.empty((B,), dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.cmt_beam_decode(self.h, src.data_ptr(), sl.data_ptr(), B, S, max_len, beam, length_penalty, eos_id,
                                             out.data_ptr(), olen.data_ptr(), osc.data_ptr()))
        return out.cpu().numpy(), olen.cpu().numpy(), osc.cpu().numpy()

    def set_regularization(self, dropout=0.0, label_smoothing=0.0, dropout_seed=0):
        """Dropout and label smoothing of the following steps (both 0 = off)."""
        self._check(self.lib.cmt_set_regularization(self.h, dropout, label_smoothing, dropout_seed))

    def time_kernel(self, name, iters):
        """(microseconds per launch, algorithmic bytes per launch) of one kernel of the last step."""
        us, nbytes = C.c_float(), C.c_double()
        self._check(self.lib.cmt_time_kernel(self.h, name.encode(), iters, C.byref(us), C.byref(nbytes)))
        return us.value, nbytes.value

    def padded_batch(self):
        return self.lib.cmt_padded_batch(self.h)

    def debug_fetch(self, name, shape):
        out = np.empty(shape, np.float32)
        self._check(self.lib.cmt_debug_fetch(self.h, name.encode(), out.ctypes.data, out.nbytes))
        return out
