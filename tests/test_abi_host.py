"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, answers the shape/byte queries bit-exactly, and rejects bad
requests before anything could be launched.  No compute call needs a GPU."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2409_11902_amd import binding as B
from paper_2409_11902_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MiB = float(1 << 20)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "cac.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b((?:cac|conv)_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert B.cac_version() == 303


def test_desc_layout_matches_header():
    hdr = open(os.path.join(ROOT, "include", "cac.h")).read()
    body = re.search(r"typedef struct cac_desc \{(.*?)\} cac_desc;", hdr, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            names += [n.strip() for n in decl.split(None, 1)[1].split(",")]
    assert names == [f[0] for f in B.cac_desc._fields_]
    assert ctypes.sizeof(B.cac_desc) == 4 * len(names)


@pytest.mark.parametrize("hw", [(56, 56), (28, 28), (14, 14), (7, 7), (5, 9), (224, 224)])
@pytest.mark.parametrize("k", [(1, 1), (2, 2), (4, 4), (2, 4), (3, 3), (5, 3)])
@pytest.mark.parametrize("mode", [B.EDGE_CEIL_VALID, B.EDGE_FLOOR_DROP])
def test_pooled_shape_bit_exact_vs_oracle(hw, k, mode):
    H, W = hw
    for dtype, eb in ((B.F32, 4), (B.BF16, 2)):
        d = B.make_desc(32, 64, 64, H, W, 3, 3, 1, 1, 1, 1, k[0], k[1], edge_mode=mode, dtype=dtype,
                        pool_mode=B.POOL_MAX if dtype == B.BF16 else B.POOL_MEAN)   # the shape does not depend on it
        hp, wp, zb, xb = B.cac_pooled_shape(d)
        assert (hp, wp) == oracle.pooled_shape(H, W, k[0], k[1], mode)
        assert (xb, zb) == oracle.saved_bytes(32, 64, H, W, k[0], k[1], eb, mode)


def test_table1_bytes_from_the_library(golden_dir):
    """Per-layer memory table, reproduced by the library's own book-keeping
    (floor/drop shapes, 4-byte elements, mini-batch 32)."""
    sums = [0.0, 0.0, 0.0]
    for line in open(os.path.join(golden_dir, "table1_memory.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "Sum":
            for mine, printed in zip(sums, map(float, f[4:7])):
                assert abs(mine - printed) <= 0.0051
            continue
        C, H, W = int(f[1]), int(f[2]), int(f[3])
        vals = []
        for k in (1, 2, 4):
            d = B.make_desc(32, C, 64, H, W, 3, 3, 1, 1, 1, 1, k, k, edge_mode=B.EDGE_FLOOR_DROP, dtype=B.F32)
            _, _, zb, xb = B.cac_pooled_shape(d)
            vals.append(zb / MiB)
            assert k != 1 or zb == xb
        for i, (mine, printed) in enumerate(zip(vals, map(float, f[4:7]))):
            assert abs(mine - printed) <= 0.0051, (f[0], vals)
            sums[i] += mine


def test_out_shape():
    for spec in sum(synth.configs().values(), []):
        d = B.desc_from_spec(spec)
        assert B.cac_out_shape(d) == (spec.P, spec.Q)


def _expect(code, fn, *a):
    with pytest.raises(B.CacError) as e:
        fn(*a)
    assert e.value.code == code, str(e.value)
    assert len(str(e.value)) > 20


def test_invalid_descriptors_are_rejected():
    good = dict(N=2, C_in=4, C_out=4, H=8, W=8, R=3, S=3, pad_h=1, pad_w=1)
    for bad in (dict(N=0), dict(C_in=-1), dict(H=0), dict(R=0), dict(stride_h=0), dict(pad_w=-1),
                dict(pool_kh=0), dict(dtype=7), dict(dw_algo=3), dict(edge_mode=3), dict(pool_mode=2), dict(pool_mode=-1),
                dict(R=11, pad_h=0)):
        d = B.make_desc(**{**good, **bad})
        _expect(B.ERR_INVALID_ARG, B.cac_pooled_shape, d)
    d = B.make_desc(**good)
    d.size = 12
    _expect(B.ERR_INVALID_ARG, B.cac_pooled_shape, d)
    rc = B.lib().cac_pooled_shape(None, None, None, None, None)
    assert rc == B.ERR_INVALID_ARG


def test_unsupported_requests():
    good = dict(N=2, C_in=4, C_out=4, H=7, W=7, R=3, S=3, pad_h=1, pad_w=1)
    _expect(B.ERR_UNSUPPORTED, B.cac_workspace_size, B.make_desc(**good, edge_mode=B.EDGE_FLOOR_DROP), B.OP_COMPRESS)
    # floor/drop is fine when the tile divides the input
    ok = B.make_desc(**{**good, "H": 8, "W": 8}, edge_mode=B.EDGE_FLOOR_DROP)
    assert B.cac_workspace_size(ok, B.OP_COMPRESS) >= 0
    _expect(B.ERR_INVALID_ARG, B.cac_workspace_size, B.make_desc(**good), 99)


def test_null_and_misaligned_pointers_fail_before_any_launch():
    """These calls would touch the GPU if validation let them through; on a
    machine without one they still return the validation error."""
    L = B.lib()
    d = B.make_desc(2, 4, 4, 8, 8, 3, 3, 1, 1, 1, 1)
    p = ctypes.byref(d)
    a = ctypes.c_void_p(0x1000)      # aligned, never dereferenced by the host
    m = ctypes.c_void_p(0x1004)      # misaligned
    assert L.conv_fwd_and_compress(p, None, a, a, a, a, None, 0, None) == B.ERR_INVALID_ARG
    assert L.conv_fwd_and_compress(p, a, a, None, a, a, None, 0, None) == B.ERR_INVALID_ARG  # has_bias, b NULL
    assert L.conv_fwd_and_compress(p, a, m, a, a, a, None, 0, None) == B.ERR_ALIGNMENT
    assert L.cac_compress(p, a, None, None) == B.ERR_INVALID_ARG
    assert L.cac_compress(p, m, a, None) == B.ERR_ALIGNMENT
    assert L.conv_bwd_weight_compressed(p, a, None, a, None, 0, None) == B.ERR_INVALID_ARG
    assert L.conv_bwd_weight_compressed(p, a, a, m, None, 0, None) == B.ERR_ALIGNMENT
    assert L.conv_bwd_data(p, None, a, a, None, 0, None) == B.ERR_INVALID_ARG
    assert L.conv_bwd_bias(p, a, None, None) == B.ERR_INVALID_ARG
    assert b"NULL" in L.cac_last_error()
    for k in range(5):
        args = [a] * 5
        args[k] = None
        assert L.conv_bwd_weight_and_data(p, *args, None, 0, None) == B.ERR_INVALID_ARG
        args[k] = m
        assert L.conv_bwd_weight_and_data(p, *args, None, 0, None) == B.ERR_ALIGNMENT
    need = B.cac_workspace_size(d, B.OP_GRAD_COSINE)
    assert need > 0
    assert L.cac_grad_cosine(p, a, None, a, a, need, None) == B.ERR_INVALID_ARG
    assert L.cac_grad_cosine(p, a, a, m, a, need, None) == B.ERR_ALIGNMENT
    assert L.cac_grad_cosine(p, a, a, a, a, need - 1, None) == B.ERR_WORKSPACE_TOO_SMALL
    assert L.cac_grad_cosine(p, a, a, a, None, 0, None) == B.ERR_WORKSPACE_TOO_SMALL


def test_workspace_too_small_is_reported():
    L = B.lib()
    for spec in (synth.configs()["cfg2_resnet18_cifar"][0], synth.configs()["cfg5_deep_small_spatial"][1]):
        d = B.desc_from_spec(spec)
        need = B.cac_workspace_size(d, B.OP_BWD_WEIGHT_COMPRESSED)
        if need == 0:
            continue
        a = ctypes.c_void_p(0x1000)
        assert L.conv_bwd_weight_compressed(ctypes.byref(d), a, a, a, a, need - 1, None) == B.ERR_WORKSPACE_TOO_SMALL
        assert L.conv_bwd_weight_compressed(ctypes.byref(d), a, a, a, None, 0, None) == B.ERR_WORKSPACE_TOO_SMALL


def test_combined_backward_workspace_holds_both_parts():
    L = B.lib()
    a = ctypes.c_void_p(0x1000)
    merged = 0
    for layers in synth.configs().values():
        for spec in layers:
            d = B.desc_from_spec(spec)
            dw, dx = B.cac_workspace_size(d, B.OP_BWD_WEIGHT_COMPRESSED), B.cac_workspace_size(d, B.OP_BWD_DATA)
            both = B.cac_workspace_size(d, B.OP_BWD_WEIGHT_AND_DATA)
            assert both == (dw + 255) // 256 * 256 + dx
            if both:
                assert L.conv_bwd_weight_and_data(ctypes.byref(d), a, a, a, a, a, a, ctypes.c_size_t(both - 1), None) == B.ERR_WORKSPACE_TOO_SMALL
            merged += "in the launch of" in B.cac_describe_plan(d, B.OP_BWD_WEIGHT_AND_DATA)
    assert merged >= 20      # most bf16 layers split their pixels and share the launch


def test_every_bf16_layer_of_the_configs_has_an_mfma_weight_gradient_plan():
    """Host-side planning only: no layer of the stated workloads falls back to the generic
    kernel, the plan's staging fits the LDS of a CU, and the workspace query covers the
    partial sums the plan announces."""
    import re
    for name, specs in synth.configs().items():
        for spec in specs:
            if spec.dtype != synth.BF16:
                continue
            d = B.desc_from_spec(spec)
            plan = B.cac_describe_plan(d, B.OP_BWD_WEIGHT_COMPRESSED)
            assert plan.startswith("dw_mfma"), (name, spec.name, plan)
            lds = int(re.search(r"lds=(\d+)B", plan).group(1))
            partial = int(re.search(r"partial=(\d+)B", plan).group(1))
            slices, tiles = map(int, re.search(r"slices=(\d+) x (\d+) tiles", plan).groups())
            assert lds <= 160 * 1024, (name, spec.name, plan)
            assert B.cac_workspace_size(d, B.OP_BWD_WEIGHT_COMPRESSED) == partial
            assert (partial == 0) == (slices == 1)
            assert slices * tiles <= 2048


def test_deep_layers_on_tiny_maps_share_out_their_channel_blocks():
    """The parity cases meant to cover the channel-split forward / data-gradient path really take it."""
    import re
    for N, C, K, H in ((4, 256, 128, 4), (6, 160, 160, 6)):
        d = B.make_desc(N, C, K, H, H, 3, 3, 1, 1, 1, 1, 2, 2, dtype=B.BF16)
        for op in (B.OP_FWD_AND_COMPRESS, B.OP_BWD_DATA):
            plan = B.cac_describe_plan(d, op)
            m = re.search(r"grid=(\d+)x(\d+)x(\d+)", plan)
            assert m and int(m.group(3)) > 1, plan
            # the float sums live in the workspace
            assert B.cac_workspace_size(d, op) >= int(m.group(3)) * N * (K if op == B.OP_FWD_AND_COMPRESS else C) * H * H * 4


def test_data_gradient_reads_dy_in_place_where_pixels_outnumber_the_filter():
    """The parity cases meant for the in-place data-gradient path take it; a filter-heavy layer does not."""
    for N, C, K, H, st in ((16, 32, 32, 16, 1), (48, 32, 32, 16, 2), (40, 24, 20, 12, 1)):
        d = B.make_desc(N, C, K, H, H, 3, 3, st, st, 1, 1, 2, 2, dtype=B.BF16)
        assert "dY read in place" in B.cac_describe_plan(d, B.OP_BWD_DATA)
    d = B.make_desc(128, 512, 512, 4, 4, 3, 3, 1, 1, 1, 1, 2, 2, dtype=B.BF16)
    assert "dY read in place" not in B.cac_describe_plan(d, B.OP_BWD_DATA)


def test_benchmark_refuses_more_than_one_gpu():
    """One GPU only: asked for more, the benchmark says so and exits before it touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout) and r.stdout.strip() == ""


def test_auto_weight_gradient_picks_by_layer_size():
    """dw_algo = AUTO: the reduced-K kernel on the large even-map 3x3 layers, the inflating one on
    small layers and wherever the reduced-K kernel does not exist (the plan string tells)."""
    cfg = synth.configs()
    def plan(spec, algo):
        return B.cac_describe_plan(B.desc_from_spec(spec, dw_algo=algo), B.OP_BWD_WEIGHT_COMPRESSED)
    big, odd = cfg["cfg5_deep_small_spatial"]
    assert plan(big, B.DW_AUTO).startswith("dw_rk") and plan(big, B.DW_AUTO) == plan(big, B.DW_REDUCED_K)
    assert plan(odd, B.DW_AUTO) == plan(odd, B.DW_INFLATE)
    small = cfg["cfg2_resnet18_cifar"][1]
    assert plan(small, B.DW_REDUCED_K).startswith("dw_rk")
    assert plan(small, B.DW_AUTO) == plan(small, B.DW_INFLATE)
    for algo in (B.DW_INFLATE, B.DW_AUTO):
        d = B.desc_from_spec(small, dw_algo=algo)
        assert B.dw_rk_executed_flops(d) == small.dw_flops
    d = B.desc_from_spec(big, dw_algo=B.DW_AUTO)
    assert B.dw_rk_executed_flops(d) * 4 == big.dw_flops
    assert B.cac_workspace_size(d, B.OP_BWD_WEIGHT_COMPRESSED) == \
        B.cac_workspace_size(B.desc_from_spec(big, dw_algo=B.DW_REDUCED_K), B.OP_BWD_WEIGHT_COMPRESSED)


def test_probe_validates_before_launching():
    """cac_probe: kind, pointers, size and iteration count are checked on the host."""
    L = B.lib()
    buf = ctypes.create_string_buffer(96)          # never dereferenced: every call below is refused
    p = ctypes.c_void_p((ctypes.addressof(buf) + 15) & ~15)
    assert L.cac_probe(5, p, p, ctypes.c_size_t(1 << 20), 1, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(-1, p, p, ctypes.c_size_t(1 << 20), 1, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(B.PROBE_COPY, None, p, ctypes.c_size_t(1 << 20), 0, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(B.PROBE_COPY, p, None, ctypes.c_size_t(1 << 20), 0, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(B.PROBE_COPY, p, p, ctypes.c_size_t(8192), 0, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(B.PROBE_COPY, p, p, ctypes.c_size_t((1 << 20) + 8), 0, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(B.PROBE_MFMA, p, p, ctypes.c_size_t(1 << 20), -1, None) == B.ERR_INVALID_ARG
    assert L.cac_probe(B.PROBE_MFMA, p, p, ctypes.c_size_t(1 << 20), (1 << 24) + 1, None) == B.ERR_INVALID_ARG
    assert b"iters" in L.cac_last_error()


def test_bn_backward_workspace_and_validation():
    """Few channels are shared out over slices (partial sums in the workspace), many are not; the
    call refuses a missing workspace before launching anything."""
    few = B.make_desc(64, 64, 8, 56, 56, 1, 1, 1, 1, 0, 0, 2, 2)
    many = B.make_desc(8, 4096, 8, 14, 14, 1, 1, 1, 1, 0, 0, 2, 2)
    odd_tile = B.make_desc(8, 64, 8, 15, 15, 1, 1, 1, 1, 0, 0, 3, 3)
    n = B.cac_workspace_size(few, B.OP_BN_BWD)
    assert n == 2 * 64 * 32 * 4                      # 2048 blocks / 64 channels = 32 slices, two sums each
    assert B.cac_workspace_size(many, B.OP_BN_BWD) == 0 and B.cac_workspace_size(odd_tile, B.OP_BN_BWD) == 0
    buf = ctypes.create_string_buffer(96)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 15) & ~15)
    L = B.lib()
    rc = L.cac_bn_bwd_compressed(ctypes.byref(few), p, p, p, p, p, p, p, p, None, 0, None)
    assert rc == B.ERR_WORKSPACE_TOO_SMALL
    rc = L.cac_bn_bwd_compressed(ctypes.byref(few), p, p, p, p, p, p, p, p, p, n - 16, None)
    assert rc == B.ERR_WORKSPACE_TOO_SMALL
    rc = L.cac_bn_bwd_compressed(ctypes.byref(few), p, None, p, p, p, p, p, p, p, n, None)
    assert rc == B.ERR_INVALID_ARG
