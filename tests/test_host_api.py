"""Host-side logic of the C-ABI library (no GPU needed): the library loads, exports every
symbol the header declares, derives tree depths / masks like the oracle does, and turns bad
arguments into status codes before anything would be launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import verify_oracle as vo
from paper_2507_22424_amd import binding as sv
from paper_2507_22424_amd import workload as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    declared = set()
    for name in ("specvla_verify.h", "specvla_verify_aux.h"):       # the path, and the measurement aids
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(sv_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sv.EXPORTS)
    lib = sv.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    assert "gfx950" in sv.sv_version()
    assert sv.sv_strerror(0) == "ok" and "tree" in sv.sv_strerror(-3)


def test_tree_masks_match_the_oracle_derivation():
    rng = np.random.default_rng(0)
    for T, dmax, kids in [(1, 7, 3), (15, 7, 3), (60, 7, 4), (64, 7, 4), (65, 9, 5), (128, 7, 6)]:
        B = 3
        parents = np.concatenate([wl.draft_tree(T, dmax, kids, min(dmax, T - 1), rng)
                                  for _ in range(B)])
        depth, anc = sv.sv_tree_build_masks(parents, B, T, dmax)
        W = (T + 63) // 64
        anc = anc.reshape(B, T, W)
        for b in range(B):
            d_ref, a_ref = vo.tree_structure(parents[b * T:(b + 1) * T])
            assert depth[b * T:(b + 1) * T].tolist() == d_ref.tolist()
            for i in range(T):
                bits = [(int(anc[b, i, j // 64]) >> (j % 64)) & 1 for j in range(T)]
                assert bits == a_ref[i].astype(int).tolist()


@pytest.mark.parametrize("parent", [[0, 0], [-1, 1], [-1, -1], [-1, 0, 3, 1], [-1, 0, 2]])
def test_bad_trees_are_rejected(parent):
    with pytest.raises(sv.SvError) as e:
        sv.sv_tree_build_masks(np.array(parent), 1, len(parent), 7)
    assert e.value.status == -3


def test_depth_cap_and_size_limits():
    chain = np.arange(-1, 9)
    with pytest.raises(sv.SvError) as e:
        sv.sv_tree_build_masks(chain, 1, 10, 7)
    assert e.value.status == -3
    sv.sv_tree_build_masks(chain, 1, 10, 9)
    with pytest.raises(sv.SvError) as e:
        sv.sv_tree_build_masks(np.arange(-1, 128), 1, 129, 31)
    assert e.value.status == -2


def test_sizes_and_cfg_checks():
    c7 = sv.model_cfg("bf16", 4096, 32, 128, 11008, 32000)
    nbytes = sv.sv_packed_layer_bytes(c7)
    weights = (4 * 4096 * 4096 + 3 * 4096 * 11008) * 2
    assert weights <= nbytes <= weights + 2 * 4096 * 4 + 8 * 256
    assert sv.sv_workspace_bytes(c7, 1, 60, 256) > 64 * 22016 * 4
    assert sv.sv_workspace_bytes(c7, 16, 60, 256) > sv.sv_workspace_bytes(c7, 1, 60, 256)
    off, nb = sv.sv_workspace_region(c7, 1, 60, 256, sv.SV_WS_ATTN_OUT)
    assert off % 256 == 0 and nb == 60 * 4096 * 4
    for bad, status in [(sv.model_cfg(5, 256, 4, 64, 688, 512), -6),
                        (sv.model_cfg("bf16", 4000, 32, 128, 11008, 32000), -2),
                        (sv.model_cfg("bf16", 4096, 64, 64, 11008, 32000), -2),
                        (sv.model_cfg("f32", 256, 4, 63, 688, 512), -2),
                        (sv.model_cfg("f32", 256, 4, 256, 688, 512), -2)]:
        with pytest.raises(sv.SvError) as e:
            sv.sv_packed_layer_bytes(bad)
        assert e.value.status == status
    with pytest.raises(sv.SvError) as e:
        sv.sv_workspace_bytes(c7, 1, 129, 256)
    assert e.value.status == -2


def test_null_and_range_arguments_fail_before_any_launch():
    lib = sv.lib()
    c1 = sv.model_cfg("f32", 256, 4, 64, 688, 512)
    assert lib.sv_verify_layer(C.byref(c1), None, None, None, None, 1, None, 0, None) == -1
    assert lib.sv_action_head_argmax(C.byref(c1), None, None, None, 1, 256, 512, None, None,
                                     None, 0, None) == -1
    assert lib.sv_pack_layer(C.byref(c1), None, None, 0, None) == -1
    assert lib.sv_relaxed_accept(None, None, None, 0, 256, 0, 1, 7, None, None, None, None,
                                 None, None) == -1
    # non-null dummies (never dereferenced on the host): range errors come first
    one = C.c_void_p(256)
    tree = sv.Tree(256, 256, 256, 15, 1)
    args = (one, one, one, one, one, None)
    assert lib.sv_relaxed_accept(C.byref(tree), one, one, 256, 256, -1, 1, 7, *args) == -4
    assert lib.sv_relaxed_accept(C.byref(tree), one, one, 256, 0, 0, 1, 7, *args) == -4
    assert lib.sv_relaxed_accept(C.byref(tree), one, one, 256, 256, 0, 0, 7, *args) == -2
    assert lib.sv_relaxed_accept(C.byref(tree), one, one, 256, 256, 0, 1, 40, *args) == -2
    bad_tree = sv.Tree(256, 256, 256, 15, 2)
    assert lib.sv_relaxed_accept(C.byref(bad_tree), one, one, 256, 256, 0, 1, 7, *args) == -2
    kv = sv.KvView(256, 256, 256, 64, 70)          # capacity < prefix + T
    assert lib.sv_verify_layer(C.byref(c1), one, one, C.byref(kv), C.byref(tree), 1, one,
                               1 << 30, None) == -2
    kv = sv.KvView(256, 256, 256, 64, 128)
    assert lib.sv_verify_layer(C.byref(c1), one, one, C.byref(kv), C.byref(tree), 1, one,
                               16, None) == -5     # workspace too small
    assert lib.sv_action_head_argmax(C.byref(c1), one, one, one, 15, 300, 200, one, None, one,
                                     1 << 30, None) == -2


def test_stack_calls_check_their_arguments_before_any_launch():
    lib = sv.lib()
    c7 = sv.model_cfg("bf16", 4096, 32, 128, 11008, 32000)
    one = C.c_void_p(256)
    tree = sv.Tree(256, 256, 256, 60, 1)
    ptrs = (C.c_void_p * 2)(256, 512)
    kvs = (sv.KvView * 2)(sv.KvView(256, 256, 256, 280, 384), sv.KvView(256, 256, 256, 280, 384))
    big = 1 << 40
    for fn, tail in ((lib.sv_verify_stack, ()),):
        assert fn(C.byref(c7), 2, None, one, kvs, C.byref(tree), 1, one, big, None, *tail) == -1
        assert fn(C.byref(c7), 0, ptrs, one, kvs, C.byref(tree), 1, one, big, None, *tail) == -2
        assert fn(C.byref(c7), 2, ptrs, one, kvs, C.byref(tree), 1, one, 16, None, *tail) == -5
        bad = (C.c_void_p * 2)(256, 0)
        assert fn(C.byref(c7), 2, bad, one, kvs, C.byref(tree), 1, one, big, None, *tail) == -1
        odd = (C.c_void_p * 2)(256, 513)          # packed blobs are 256-byte aligned
        assert fn(C.byref(c7), 2, odd, one, kvs, C.byref(tree), 1, one, big, None, *tail) == -5


def test_eight_bit_weight_packing_checks_its_arguments_before_any_launch():
    """SV_BF16_W8: half the matrix bytes plus the row scales; the two pack calls each refuse the
    other's dtype; nothing is launched on bad arguments."""
    lib = sv.lib()
    bf = sv.model_cfg("bf16", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    w8 = sv.model_cfg("bf16_w8", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    nb, n8 = sv.sv_packed_layer_bytes(bf), sv.sv_packed_layer_bytes(w8)
    H, D, F = 512, 512, 1536
    matrix_elems = 3 * D * H + H * D + 2 * F * H + H * F
    assert nb - n8 >= matrix_elems - 4 * (3 * D + 2 * H + 2 * F) - 8 * 256      # 1 byte less per element, scales added
    assert n8 >= matrix_elems + 4 * (3 * D + 2 * H + 2 * F)
    one = C.c_void_p(256)
    raw = sv.LayerWeights(*([256] * 9))
    sc = sv.LayerScales(*([256] * 7))
    assert lib.sv_pack_layer_w8(C.byref(bf), C.byref(raw), C.byref(sc), one, 1 << 30, None) == -6
    assert lib.sv_pack_layer(C.byref(w8), C.byref(raw), one, 1 << 30, None) == -6
    assert lib.sv_pack_layer_w8(C.byref(w8), None, C.byref(sc), one, 1 << 30, None) == -1
    assert lib.sv_pack_layer_w8(C.byref(w8), C.byref(raw), None, one, 1 << 30, None) == -1
    no_scale = sv.LayerScales(256, 256, 256, 256, 256, 256, None)
    assert lib.sv_pack_layer_w8(C.byref(w8), C.byref(raw), C.byref(no_scale), one, 1 << 30, None) == -1
    assert lib.sv_pack_layer_w8(C.byref(w8), C.byref(raw), C.byref(sc), one, n8 - 1, None) == -5
    assert lib.sv_pack_layer_w8(C.byref(w8), C.byref(raw), C.byref(sc), C.c_void_p(260), n8, None) == -5
    odd = sv.model_cfg("bf16_w8", 384, 4, 128, 1536, 1024, 1e-5, 10000.0)      # hidden not a multiple of 256
    assert lib.sv_pack_layer_w8(C.byref(odd), C.byref(raw), C.byref(sc), one, 1 << 30, None) == -2


def test_four_bit_weight_packing_checks_its_arguments_before_any_launch():
    """SV_BF16_W4: a quarter of the bf16 matrix bytes plus the row scales; each pack call refuses
    the dtypes of the others; nothing is launched on bad arguments."""
    lib = sv.lib()
    bf = sv.model_cfg("bf16", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    w8 = sv.model_cfg("bf16_w8", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    w4 = sv.model_cfg("bf16_w4", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    n8, n4 = sv.sv_packed_layer_bytes(w8), sv.sv_packed_layer_bytes(w4)
    H, D, F = 512, 512, 1536
    matrix_elems = 3 * D * H + H * D + 2 * F * H + H * F
    scales = 4 * (3 * D + 2 * H + 2 * F)
    assert matrix_elems // 2 + scales <= n4 <= matrix_elems // 2 + scales + 2 * 512 * 4 + 12 * 256
    assert n8 - n4 >= matrix_elems // 2 - 8 * 256
    one = C.c_void_p(256)
    raw = sv.LayerWeights(*([256] * 9))
    sc = sv.LayerScales(*([256] * 7))
    assert lib.sv_pack_layer_w4(C.byref(bf), C.byref(raw), C.byref(sc), one, 1 << 30, None) == -6
    assert lib.sv_pack_layer_w4(C.byref(w8), C.byref(raw), C.byref(sc), one, 1 << 30, None) == -6
    assert lib.sv_pack_layer_w8(C.byref(w4), C.byref(raw), C.byref(sc), one, 1 << 30, None) == -6
    assert lib.sv_pack_layer(C.byref(w4), C.byref(raw), one, 1 << 30, None) == -6
    assert lib.sv_pack_layer_w4(C.byref(w4), None, C.byref(sc), one, 1 << 30, None) == -1
    assert lib.sv_pack_layer_w4(C.byref(w4), C.byref(raw), None, one, 1 << 30, None) == -1
    assert lib.sv_pack_layer_w4(C.byref(w4), C.byref(raw), C.byref(sc), one, n4 - 1, None) == -5
    assert lib.sv_pack_layer_w4(C.byref(w4), C.byref(raw), C.byref(sc), C.c_void_p(260), n4, None) == -5
    odd = sv.model_cfg("bf16_w4", 384, 4, 128, 1536, 1024, 1e-5, 10000.0)      # hidden not a multiple of 256
    assert lib.sv_pack_layer_w4(C.byref(odd), C.byref(raw), C.byref(sc), one, 1 << 30, None) == -2


def test_packed_head_checks_its_arguments_before_any_launch():
    """Packed head: gain + rows in bytes; bf16 only; scored range a multiple of 32 inside the
    vocabulary; buffers aligned and large enough; workspace grows with the scored rows."""
    lib = sv.lib()
    bf = sv.model_cfg("bf16", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    f32 = sv.model_cfg("f32", 512, 4, 128, 1536, 1024, 1e-5, 10000.0)
    nb = sv.sv_packed_head_bytes(bf, 768, 1024)
    assert 256 * 512 * 2 + 512 * 4 <= nb <= 256 * 512 * 2 + 512 * 4 + 512
    assert sv.sv_packed_head_bytes(bf, 0, 1024) >= 1024 * 512 * 2 + 512 * 4
    out = C.c_size_t(0)
    one = C.c_void_p(256)
    assert lib.sv_packed_head_bytes(C.byref(f32), 768, 1024, C.byref(out)) == -6
    assert lib.sv_packed_head_bytes(C.byref(bf), 768, 1024, None) == -1
    for lo, hi in ((768, 1000), (-32, 0), (1024, 1024), (1000, 1056), (512, 480)):
        assert lib.sv_packed_head_bytes(C.byref(bf), lo, hi, C.byref(out)) == -2, (lo, hi)
        assert lib.sv_pack_head(C.byref(bf), one, one, lo, hi, one, 1 << 30, None) == -2
        assert lib.sv_action_head_argmax_packed(C.byref(bf), one, one, 4, lo, hi, one, None, one,
                                                1 << 40, None) == -2
    assert lib.sv_pack_head(C.byref(f32), one, one, 768, 1024, one, 1 << 30, None) == -6
    assert lib.sv_pack_head(C.byref(bf), None, one, 768, 1024, one, 1 << 30, None) == -1
    assert lib.sv_pack_head(C.byref(bf), one, None, 768, 1024, one, 1 << 30, None) == -1
    assert lib.sv_pack_head(C.byref(bf), one, one, 768, 1024, None, 1 << 30, None) == -1
    assert lib.sv_pack_head(C.byref(bf), one, one, 768, 1024, one, nb - 1, None) == -5
    assert lib.sv_pack_head(C.byref(bf), one, one, 768, 1024, C.c_void_p(264), nb, None) == -5
    ws = sv.sv_workspace_bytes(bf, 1, 8, 256)
    assert ws > sv.sv_workspace_bytes(bf, 1, 8, 0)
    assert sv.sv_workspace_bytes(bf, 1, 8, 1024) > ws
    args = (C.byref(bf), one, one, 8, 768, 1024, one, None, one)
    assert lib.sv_action_head_argmax_packed(*args, ws - 1, None) == -5
    assert lib.sv_action_head_argmax_packed(C.byref(bf), one, one, 8, 768, 1024, one, None,
                                            C.c_void_p(264), ws, None) == -5
    assert lib.sv_action_head_argmax_packed(C.byref(bf), C.c_void_p(264), one, 8, 768, 1024, one,
                                            None, one, ws, None) == -5
    assert lib.sv_action_head_argmax_packed(C.byref(bf), None, one, 8, 768, 1024, one, None, one,
                                            ws, None) == -1
    assert lib.sv_action_head_argmax_packed(C.byref(bf), one, one, 0, 768, 1024, one, None, one,
                                            ws, None) == -2
    assert lib.sv_action_head_argmax_packed(C.byref(f32), one, one, 8, 768, 1024, one, None, one,
                                            ws, None) == -6


def test_stream_read_checks_its_arguments_before_any_launch():
    lib = sv.lib()
    a = C.c_void_p(4096)
    assert lib.sv_stream_read(None, 4096, a, None) == -1
    assert lib.sv_stream_read(a, 4096, None, None) == -1
    assert lib.sv_stream_read(a, 0, a, None) == -2
    assert lib.sv_stream_read(a, 4100, a, None) == -2
    assert lib.sv_stream_read(C.c_void_p(4100), 4096, a, None) == -2
    assert lib.sv_stream_read(a, 4096, C.c_void_p(4104), None) == -2


def test_bench_refuses_more_than_one_gpu_with_a_message():
    """Nothing here uses a second GPU: `bench.py --gpus N` with N > 1 exits with a message (before
    anything touches a GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "--gpus must be 1" in (r.stderr + r.stdout)
