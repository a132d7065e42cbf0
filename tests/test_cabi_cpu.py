"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-only logic (configuration validation, size queries) behaves.  No compute call is made."""
import ctypes as C
import os
import re

import pytest

from paper_1802_07170_amd import binding, inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1802_07170_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cytonmt_hip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cmt_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_query_sizes_for_the_five_workloads(lib):
    for name, c in I.CONFIGS.items():
        cfg = I.model_cfg(c)
        cc = binding.make_config(cfg, c["batch"], c["len_range"][1], c["len_range"][1], c["precision"])
        pb, gb, wb = binding.query_sizes(cc)
        assert pb == gb == 4 * I.param_count(cfg), name
        assert wb > 0 and wb % 256 == 0
        assert wb < 64 * 2 ** 30, (name, wb)            # far below the 288 GB of one MI355X


def test_unsupported_configurations_are_rejected(lib):
    good = dict(src_vocab=1000, tgt_vocab=1000, emb=64, hidden=64, layers=1)
    def rc(cfg=good, **kw):
        args = dict(max_batch=8, max_src_len=10, max_tgt_len=10, precision=0)
        args.update(kw)
        cc = binding.make_config(cfg, **args)
        a = C.c_size_t()
        return lib.cmt_query_sizes(C.byref(cc), C.byref(a), C.byref(a), C.byref(a))
    assert rc() == binding.CMT_OK
    assert rc(dict(good, hidden=72)) == binding.CMT_EINVAL          # hidden not a multiple of 16
    assert rc(dict(good, hidden=2048)) == binding.CMT_EINVAL        # beyond the kernels' register tiling
    assert rc(dict(good, emb=12)) == binding.CMT_EINVAL
    assert rc(dict(good, tgt_vocab=1001)) == binding.CMT_EINVAL
    assert rc(dict(good, layers=0)) == binding.CMT_EINVAL
    assert rc(precision=2) == binding.CMT_EINVAL
    assert rc(max_batch=0) == binding.CMT_EINVAL
    assert rc(max_src_len=513) == binding.CMT_EINVAL
    assert rc(bos_id=1000) == binding.CMT_EINVAL
    assert lib.cmt_query_sizes(None, None, None, None) == binding.CMT_EINVAL


def test_create_rejects_null_and_misaligned_buffers(lib):
    cc = binding.make_config(dict(src_vocab=1000, tgt_vocab=1000, emb=64, hidden=64, layers=1), 8, 10, 10, 0)
    h = C.c_void_p()
    assert lib.cmt_create(C.byref(cc), None, None, None, None, C.byref(h)) == binding.CMT_EINVAL
    assert lib.cmt_create(C.byref(cc), 256, 512, 100, None, C.byref(h)) == binding.CMT_EINVAL   # misaligned
    assert not h.value
    assert lib.cmt_param_count(None) == binding.CMT_EINVAL
    assert lib.cmt_last_error(None) == b"null handle"


def test_workload_generators_follow_the_recipe():
    import numpy as np
    c = I.CONFIGS["medium"]
    src, sl, tgt, tl = I.make_batch(c)
    assert src.shape == (64, sl.max()) and tgt.shape == (64, tl.max())
    assert sl.min() >= 20 and sl.max() <= 50 and tl.min() >= 20 and tl.max() <= 50
    for ids, ln in ((src, sl), (tgt, tl)):
        valid = np.arange(ids.shape[1])[None] < ln[:, None]
        assert ids[valid].min() >= 4 and ids[valid].max() < c["src_vocab"]
        assert (ids[~valid] == I.PAD_ID).all()
    # bounded Zipf(1.1): p(rank k) = k^-1.1 / sum_{k=1}^{V-4} k^-1.1; rank 1 is id 4
    ids = I.zipf_ids(np.random.default_rng(0), 32000, 200000)
    frac = (ids == 4).mean()
    p1 = 1.0 / (np.arange(1, 32000 - 3, dtype=np.float64) ** -1.1).sum()
    assert abs(frac - p1) < 0.005 and 0.13 < p1 < 0.15
    assert ids.min() == 4 and ids.max() < 32000
    assert (np.bincount(ids)[4:8] > np.bincount(ids)[100:104]).all()
    again = I.make_batch(c)
    assert all(np.array_equal(a, b) for a, b in zip((src, sl, tgt, tl), again))
    t = I.CONFIGS["tiny"]
    s2, sl2, _, _ = I.make_batch(t)
    assert s2.shape == (8, 10) and (sl2 == 10).all()


C_PROGRAM = r"""
#include <stdio.h>
#include "cytonmt_hip.h"
int main(void) {
  cmt_config c;
  size_t pb = 0, gb = 0, wb = 0;
  c.src_vocab = 1000; c.tgt_vocab = 1000; c.emb_dim = 64; c.hidden = 64; c.layers = 1;
  c.max_batch = 8; c.max_src_len = 10; c.max_tgt_len = 10; c.precision = 0; c.bos_id = 2; c.pad_id = 0;
  if (cmt_query_sizes(&c, &pb, &gb, &wb) != CMT_OK) return 1;
  c.hidden = 65;
  if (cmt_query_sizes(&c, &pb, &gb, &wb) != CMT_EINVAL) return 2;
  printf("%zu %zu %zu\n", pb, gb, wb);
  return 0;
}
"""


def test_header_is_plain_c_and_a_c_program_links_against_the_library(lib, tmp_path):
    """The boundary is usable without Python or C++: the header compiles as C99 (pedantic) and as C++,
    and a C program linked against the library calls a host-only entry point."""
    import shutil
    import subprocess
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "prog.c"
    src.write_text(C_PROGRAM)
    exe = tmp_path / "prog"
    libdir = os.path.dirname(binding.LIB_PATH)
    rocm_lib = "/opt/rocm/lib"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe),
                    "-L", libdir, "-lcytonmt_hip", f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{rocm_lib}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    cfg = I.model_cfg(I.CONFIGS["tiny"])
    assert int(out[0]) == int(out[1]) == 4 * I.param_count(cfg) and int(out[2]) > 0
    if shutil.which("g++"):
        cpp = tmp_path / "prog.cpp"
        cpp.write_text('#include "cytonmt_hip.h"\nint main() { return cmt_param_count(nullptr) == CMT_EINVAL ? 0 : 1; }\n')
        subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)], check=True)
