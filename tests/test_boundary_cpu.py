"""Host-only checks of the C-ABI boundary: the library loads, exports what the header declares, and
rejects bad configurations before touching any device (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2205_05632_amd import binding as B
from paper_2205_05632_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "compams.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(compams_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in names:
        assert hasattr(L, name), name


def test_header_compiles_as_plain_c(tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "compams.h"\nint main(void){compams_config c; (void)c; return COMPAMS_OK;}\n')
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c", str(src),
                    "-o", str(tmp_path / "t.o")], check=True)


def test_binding_struct_matches_the_header(tmp_path):
    """Size of compams_config and the offset of every field, as a C compiler lays out the header's struct."""
    fields = [f[0] for f in B.compams_config._fields_]
    src = tmp_path / "layout.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "compams.h"', 'int main(void){',
             'printf("%zu\\n", sizeof(compams_config));']
    lines += [f'printf("%zu\\n", offsetof(compams_config, {f}));' for f in fields]
    lines += ['return 0;}']
    src.write_text("\n".join(lines))
    import subprocess
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(B.compams_config)
    assert out[1:] == [getattr(B.compams_config, f).offset for f in fields]
    text = open(os.path.join(ROOT, "include", "compams.h")).read()
    for name, value in (("NONE", B.NONE), ("TOPK", B.TOPK), ("BLOCKSIGN", B.BLOCKSIGN), ("TOPK_BLOCKS", B.TOPK_BLOCKS)):
        assert re.search(rf"COMPAMS_{name}\s*=\s*{value}\b", text), name
    for name, value in B.STATE.items():       # the queries of compams_state
        assert re.search(rf"COMPAMS_STATE_{name.upper()}\s*=\s*{value}\b", text), name


def cfg(**kw):
    c = B.compams_config()
    c.n, c.d, c.ld, c.compressor, c.k = 4, 1000, 1000, B.TOPK, 10
    c.beta1, c.beta2, c.eps = 0.9, 0.999, 1e-8
    fake = 0x1000  # never dereferenced: validation fails first
    c.theta = c.m = c.v = c.vhat = c.e = c.workspace = fake
    c.workspace_bytes = 1 << 40
    for k_, v_ in kw.items():
        setattr(c, k_, v_)
    return c


def test_workspace_size_is_host_only_and_monotone():
    L = B.lib()
    base = L.compams_workspace_size(ctypes.byref(cfg()))
    assert base > 0 and base % 256 == 0
    assert L.compams_workspace_size(ctypes.byref(cfg(k=500))) > base
    assert L.compams_workspace_size(ctypes.byref(cfg(n=0))) == 0
    assert L.compams_workspace_size(ctypes.byref(cfg(k=0))) == 0
    assert L.compams_workspace_size(ctypes.byref(cfg(k=1001))) == 0
    assert L.compams_workspace_size(ctypes.byref(cfg(d=1 << 31))) == 0
    assert L.compams_workspace_size(ctypes.byref(cfg(compressor=7))) == 0
    assert L.compams_workspace_size(None) == 0
    # headline configuration: well under a GiB of scratch
    w = W.get("r18_topk1")
    c = cfg(n=w.n, d=w.d, ld=B.padded_ld(w.d), k=w.k)
    assert 0 < L.compams_workspace_size(ctypes.byref(c)) < (1 << 30)


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), -1), (dict(n=65536), -1), (dict(d=0), -1), (dict(k=0), -1), (dict(k=1001), -1), (dict(ld=996), -1),
    (dict(ld=1002), -2), (dict(eps_mode=5), -1), (dict(theta=None), -1), (dict(workspace=None), -1),
    (dict(theta=0x1004), -2), (dict(workspace=0x1010), -2), (dict(workspace_bytes=16), -3),
    (dict(compressor=B.BLOCKSIGN, num_blocks=2), -1),      # no offsets given
])
def test_init_rejects_bad_configs_without_touching_the_device(kw, code):
    h = ctypes.c_void_p()
    assert B.lib().compams_init(ctypes.byref(cfg(**kw)), ctypes.byref(h)) == code
    assert not h.value


def test_init_rejects_bad_block_offsets():
    for off in ([1, 5, 1000], [0, 5, 5, 1000], [0, 5, 999], [0, 600, 500, 1000]):
        a = np.array(off, dtype=np.int64)
        c = cfg(compressor=B.BLOCKSIGN, num_blocks=len(off) - 1)
        c.block_offsets = a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        h = ctypes.c_void_p()
        assert B.lib().compams_init(ctypes.byref(c), ctypes.byref(h)) == -1


def blocks_cfg(off, kb, **kw):
    a = np.array(off, dtype=np.int64)
    b = np.array(kb, dtype=np.int64)
    c = cfg(compressor=B.TOPK_BLOCKS, k=0, num_blocks=len(off) - 1, **kw)
    c.block_offsets = a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    if kb is not None and len(kb):
        c.block_k = b.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    c._keep = (a, b)
    return c


def test_topk_inside_blocks_is_validated_on_the_host():
    L = B.lib()
    good = blocks_cfg([0, 400, 1000], [4, 6])
    size = L.compams_workspace_size(ctypes.byref(good))
    assert size > 0 and size % 256 == 0
    k = 10
    assert L.compams_wire_capacity(ctypes.byref(good)) == 3 + ((k + 255) // 256 + 3) // 4 + 2 * k
    assert L.compams_workspace_size(ctypes.byref(blocks_cfg([0, 400, 1000], [40, 60]))) > size
    for off, kb in (([0, 400, 1000], [401, 1]), ([0, 400, 1000], [0, 1]), ([0, 400, 999], [1, 1]),
                    ([0, 400, 400, 1000], [1, 1, 1]), ([4, 400, 1000], [1, 1]), ([0, 400, 1000], [])):
        c = blocks_cfg(off, kb)
        assert L.compams_workspace_size(ctypes.byref(c)) == 0, (off, kb)
        assert L.compams_wire_capacity(ctypes.byref(c)) == 0
        h = ctypes.c_void_p()
        assert L.compams_init(ctypes.byref(c), ctypes.byref(h)) == -1 and not h.value
    h = ctypes.c_void_p()
    assert L.compams_init(ctypes.byref(blocks_cfg([0, 402, 1000], [1, 1])), ctypes.byref(h)) == -2  # 402 % 4 != 0
    assert L.compams_init(ctypes.byref(blocks_cfg([0, 400, 1000], [4, 6], workspace_bytes=256)), ctypes.byref(h)) == -3
    assert not h.value
    # the per-layer workload: scratch stays well under a GiB
    w = W.get("r18_topk1_layers")
    c = blocks_cfg(w.block_offsets(), w.block_k(), n=w.n, d=w.d, ld=B.padded_ld(w.d))
    assert 0 < L.compams_workspace_size(ctypes.byref(c)) < (1 << 30)


def test_null_context_is_rejected_everywhere():
    L = B.lib()
    assert L.compams_step(None, 0x1000, 1e-3, None) == -1
    assert L.compams_destroy(None) == -1
    assert L.compams_set_option(None, 0, 0) == -1
    assert L.compams_set_option(None, B.OPT_CACHED_ARRAYS, 2) == -1
    assert L.compams_profile_enable(None, 1) == -1
    p, c = ctypes.c_void_p(), ctypes.c_int64()
    assert L.compams_state(None, 0, ctypes.byref(p), ctypes.byref(c)) == -1
    assert L.compams_copy(None, None, 16, None) == -1
    assert L.compams_copy(0x1000, 0x2000, 8, None) == -2
    assert L.compams_inplace_probe((ctypes.c_void_p * 2)(0x1000, 0x2000), 2, 16, 5, None) == -1
    assert L.compams_cached_state_arrays(0) == -1
    # the workloads' sizes: four arrays of 45 MB all fit, of 102 MB two, of 498 MB none
    assert [B.compams_cached_state_arrays(d) for d in (1, 11181642, 25557032, 124439808)] == [4, 4, 2, 0]
    two = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    assert L.compams_inplace_probe(None, 1, 16, 0, None) == -1
    assert L.compams_inplace_probe(two, 5, 16, 0, None) == -1
    assert L.compams_inplace_probe(two, 2, 6, 0, None) == -2
    assert L.compams_inplace_probe((ctypes.c_void_p * 2)(0x1000, 0x2004), 2, 16, 0, None) == -2


def test_strerror_covers_every_status():
    seen = {B.compams_strerror(s) for s in range(0, -6, -1)}
    assert len(seen) == 6 and "unknown status" not in seen
    assert B.compams_strerror(-99) == "unknown status"


def test_workload_shapes_match_the_named_models():
    assert (len(W.resnet18_shapes()), sum(W.resnet18_shapes())) == (62, 11181642)
    assert (len(W.resnet50_shapes()), sum(W.resnet50_shapes())) == (161, 25557032)
    assert (len(W.gpt2_small_shapes()), sum(W.gpt2_small_shapes())) == (148, 124439808)
    assert W.get("r18_topk1").k == 111816 and W.get("r18_topk01").k == 11181
    assert W.get("r50_topk1").k == 255570 and W.get("gpt2s_topk01").k == 124439
    off = W.get("gpt2s_blocksign").block_offsets()
    assert len(off) - 1 == 30381 and off[-1] - off[-2] == 3328


def test_gradients_are_a_pure_function_of_seed_and_step():
    w = W.get("tiny")
    a, b, c = W.gradients(w, 3), W.gradients(w, 3), W.gradients(w, 4)
    assert a.equal(b) and not a.equal(c)
    w4 = W.Workload("emb", 2, [8 * 16, 40], "normal", "topk", k=4, sparse_rows=(0, 16, 0.5))
    g = W.gradients(w4, 0)
    rows = g[:, :128].view(2, 8, 16)
    zero_rows = (rows == 0).all(dim=2)
    assert zero_rows.any() and not zero_rows.all()
    assert not np.signbit(g.numpy()[g.numpy() == 0]).any()      # dropped rows are +0.0
