"""Parity of the HIP path against the CPU oracle, element by element, on the
same seeded inputs.  Every call goes through the C ABI (ctypes binding).

Tolerances (relative L2 error ||got - want|| / ||want||):
  float path    <= 1e-5   (true fp32 multiply-accumulate)
  bfloat16 path <= 2e-2   (bf16 storage incl. the stored Z, fp32 accumulation)
and, in addition, a tight check that isolates indexing from storage rounding:
the oracle is also run from its own Z rounded to bfloat16 by the harness, which
the device result must match to 2e-4 (only the summation order differs).
Shapes, byte counts: bit-exact.
"""
import numpy as np
import pytest

import oracle
from paper_2409_11902_amd import synth
from util import check_bf16_output, geom, rel_l2, tile_constant_activation

pytestmark = pytest.mark.gpu

TOL = {synth.F32: 1e-5, synth.BF16: 2e-2}
TIGHT = 2e-4


def _oracle_step(spec, t, has_bias=True):
    g = geom(spec)
    X, Wt, b, dY = (t[k].astype(np.float64) for k in ("X", "W", "b", "dY"))
    Z = oracle.avgpool(X, spec.k, spec.k)
    Xh = oracle.inflate(Z, spec.H, spec.W, spec.k, spec.k)
    return dict(Y=oracle.conv_fwd(g, X, Wt, b if has_bias else None), Z=Z, dW=oracle.conv_dw(g, Xh, dY),
                dX=oracle.conv_dx(g, Wt, dY), db=oracle.bias_grad(dY))


def _check_step(spec, t, got, has_bias=True):
    want = _oracle_step(spec, t, has_bias)
    tol = TOL[spec.dtype]
    for name in ("Y", "Z", "dW", "dX", "db"):
        assert got[name].shape == want[name].shape, name
        err = rel_l2(got[name], want[name])
        assert err <= tol, f"{spec.name} {name}: rel-L2 {err:.3e} > {tol}"
    g = geom(spec)
    if spec.dtype == synth.BF16:
        # tight: same storage rounding of Z on both sides
        Zr = synth.round_to_bf16(want["Z"].astype(np.float32)).astype(np.float64)
        ulp_off = np.abs(got["Z"] - Zr) > np.abs(Zr) * 2.0 ** -7
        assert ulp_off.mean() == 0.0, f"{spec.name}: Z differs by more than one bf16 ulp"
        dWr = oracle.conv_dw(g, oracle.inflate(Zr, spec.H, spec.W, spec.k, spec.k), t["dY"].astype(np.float64))
        err = rel_l2(got["dW"], dWr)
        assert err <= TIGHT, f"{spec.name} dW (tight): rel-L2 {err:.3e}"
        # Y and dX, every element: the oracle value rounded to bfloat16, or its neighbour
        check_bf16_output(got["Y"], want["Y"], f"{spec.name} Y")
        check_bf16_output(got["dX"], want["dX"], f"{spec.name} dX")
    else:
        err = rel_l2(got["dW"], want["dW"])
        assert err <= 1e-5


def test_config1_single_conv_fp32():
    from gpu_util import run_step
    spec = synth.configs()["cfg1_single_fp32"][0]
    t = synth.make_inputs(spec, "cfg1_single_fp32")
    got = run_step(spec, t)
    _check_step(spec, t, got)


# small shapes that still span several tiles and ragged tails; asymmetric on purpose
SMALL = [
    # name, N, C, K, H, W, R, S, stride, pad, k
    ("3x3 ragged 7", 3, 5, 6, 7, 7, 3, 3, 1, 1, 2),
    ("3x3 14 k4", 2, 8, 4, 14, 14, 3, 3, 1, 1, 4),
    ("3x3 s2 odd", 2, 6, 10, 15, 15, 3, 3, 2, 1, 2),
    ("1x1", 4, 16, 8, 8, 8, 1, 1, 1, 0, 2),
    ("1x1 s2", 4, 8, 16, 14, 14, 1, 1, 2, 0, 2),
    ("3x3 k1", 2, 4, 4, 9, 9, 3, 3, 1, 1, 1),
    ("5x5 pad2", 2, 3, 5, 12, 12, 5, 5, 1, 2, 2),
    ("3x3 nopad", 2, 4, 4, 10, 10, 3, 3, 1, 0, 2),
    ("7x7 s2 pad3", 1, 3, 8, 20, 20, 7, 7, 2, 3, 2),
    ("tiny 1px", 1, 1, 1, 1, 1, 1, 1, 1, 0, 2),
    ("k larger than map", 2, 3, 3, 3, 3, 3, 3, 1, 1, 4),
    ("wide channels", 2, 70, 33, 6, 6, 3, 3, 1, 1, 2),
    # several images per pixel tile with a ragged last group; channels not a multiple of 32
    ("4x4 maps batch 5", 5, 48, 40, 4, 4, 3, 3, 1, 1, 2),
    ("8x8 maps batch 9", 9, 64, 64, 8, 8, 3, 3, 1, 1, 2),
    ("7x7 maps batch 6", 6, 32, 96, 7, 7, 3, 3, 1, 1, 2),
    # row lengths of 1, 2, 4 and 7 eight-pixel segments (compile-time row walks) and one that is none of them
    ("row 14", 3, 32, 32, 14, 14, 3, 3, 1, 1, 2),
    ("row 28", 2, 32, 64, 28, 28, 3, 3, 1, 1, 2),
    ("row 56", 1, 16, 32, 56, 56, 3, 3, 1, 1, 4),
    ("row 40", 1, 16, 16, 40, 40, 3, 3, 1, 1, 2),
    # pixel split over the waves with an uneven number of row pairs; edge tiles in both channel dims
    ("12x12 c72 k40", 3, 72, 40, 12, 12, 3, 3, 1, 1, 2),
    ("s2 parity classes", 3, 32, 48, 16, 16, 3, 3, 2, 1, 2),
    ("1x1 wide", 2, 128, 64, 14, 14, 1, 1, 1, 0, 2),
    ("1x1 s2 wide", 2, 96, 160, 14, 14, 1, 1, 2, 0, 4),
    # 1x1 stride 2 on even maps: three of the four parity classes of the data gradient have no taps
    ("1x1 s2 even grid", 3, 40, 24, 12, 12, 1, 1, 2, 0, 2),
    ("1x1 s2 even grid wide", 2, 64, 128, 16, 24, 1, 1, 2, 0, 2),
    ("1x1 s2 even grid 5 img", 5, 32, 32, 8, 8, 1, 1, 2, 0, 2),
    ("1x1 s2 rows of 6", 2, 32, 64, 12, 6, 1, 1, 2, 0, 2),
    # few taps: four 32-channel groups per pass, the last of them partly (100 -> 112 of 128 channels) or
    # wholly (200 -> 208 of 256) beyond the tensor's channels; two groups with the four-tap class of a
    # stride-2 data gradient
    ("1x1 c100", 3, 100, 72, 10, 10, 1, 1, 1, 0, 2),
    ("1x1 c200 s2", 2, 200, 64, 8, 8, 1, 1, 2, 0, 2),
    ("3x3 s2 k112", 2, 40, 112, 12, 12, 3, 3, 2, 1, 2),
    # deep layers on tiny maps: forward and data gradient share a tile's channel blocks out over
    # several workgroups (float partial sums + a finishing pass); 160 channels = 5 blocks
    ("4x4 maps deep", 4, 256, 128, 4, 4, 3, 3, 1, 1, 2),
    ("6x6 maps c160", 6, 160, 160, 6, 6, 3, 3, 1, 1, 2),
    # many pixels per filter element: the data gradient reads dY where it lies (8 x 8 transposes in
    # its copy waves) instead of a channels-last copy; stride 2 (four classes), a row of 12 pixels
    # (a partial 8-pixel group), 20 channels (a partial channel octet)
    ("dY in place", 16, 32, 32, 16, 16, 3, 3, 1, 1, 2),
    ("dY in place s2", 48, 32, 32, 16, 16, 3, 3, 2, 1, 2),
    ("dY in place w12 k20", 40, 24, 20, 12, 12, 3, 3, 1, 1, 2),
]


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_shapes(case, dtype):
    from gpu_util import run_step
    name, N, C, K, H, W, R, S, st, pad, k = case
    spec = synth.LayerSpec(name, N, C, K, H, W, R, S, st, pad, k, dtype)
    t = synth.make_inputs(spec, "small")
    got = run_step(spec, t)
    _check_step(spec, t, got)


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_rectangular_and_anisotropic(dtype):
    """H != W, R != S, stride/pad/pooling tile different per axis (descriptor fields
    the LayerSpec shorthand does not cover)."""
    from gpu_util import run_step
    spec = synth.LayerSpec("rect", 2, 6, 5, 10, 17, 3, 3, 1, 1, 2, dtype)
    over = dict(R=3, S=2, stride_h=2, stride_w=1, pad_h=1, pad_w=0, pool_kh=2, pool_kw=4)
    g = oracle.ConvGeom(2, 6, 5, 10, 17, 3, 2, 2, 1, 1, 0)
    rng = np.random.Generator(np.random.Philox(key=77))
    t = dict(X=synth.to_storage(np.maximum(rng.standard_normal((2, 6, 10, 17), dtype=np.float32), 0), dtype),
             W=synth.to_storage(rng.standard_normal((5, 6, 3, 2), dtype=np.float32), dtype),
             b=synth.to_storage(rng.standard_normal((5,), dtype=np.float32), dtype),
             dY=synth.to_storage(rng.standard_normal((2, 5, g.P, g.Q), dtype=np.float32), dtype))
    # run_step sizes its buffers from the spec: give it one whose P, Q, R, S match
    from paper_2409_11902_amd import binding as B
    import torch
    from gpu_util import Guarded, upload, download, tdtype, workspace
    d = B.desc_from_spec(spec, **over)
    hp, wp, zb, xb = B.cac_pooled_shape(d)
    assert (hp, wp) == oracle.pooled_shape(10, 17, 2, 4) and B.cac_out_shape(d) == (g.P, g.Q)
    td = tdtype(spec)
    X, Wt, b, dY = (upload(t[k], dtype) for k in ("X", "W", "b", "dY"))
    Y, Z = Guarded((2, 5, g.P, g.Q), td), Guarded((2, 6, hp, wp), td)
    dW, dX, db = Guarded((5, 6, 3, 2), torch.float32), Guarded((2, 6, 10, 17), td), Guarded((5,), torch.float32)
    B.conv_fwd_and_compress(d, X, Wt, b, Y.t, Z.t, workspace(d, B.OP_FWD_AND_COMPRESS))
    B.conv_bwd_weight_compressed(d, Z.t, dY, dW.t, workspace(d, B.OP_BWD_WEIGHT_COMPRESSED))
    B.conv_bwd_data(d, Wt, dY, dX.t, workspace(d, B.OP_BWD_DATA))
    B.conv_bwd_bias(d, dY, db.t)
    torch.cuda.synchronize()
    for gb in (Y, Z, dW, dX, db):
        gb.check("rect")
    f = {k: v.astype(np.float64) for k, v in t.items()}
    Zo = oracle.avgpool(f["X"], 2, 4)
    want = dict(Y=oracle.conv_fwd(g, f["X"], f["W"], f["b"]), Z=Zo,
                dW=oracle.conv_dw(g, oracle.inflate(Zo, 10, 17, 2, 4), f["dY"]),
                dX=oracle.conv_dx(g, f["W"], f["dY"]), db=oracle.bias_grad(f["dY"]))
    got = dict(Y=Y, Z=Z, dW=dW, dX=dX, db=db)
    for name in want:
        err = rel_l2(download(got[name].t), want[name])
        assert err <= TOL[dtype], f"{name}: {err:.3e}"


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_invariants_on_device(dtype):
    """k = 1 stores X itself; Y and dX do not depend on k (they never see Z);
    a tile-constant activation is compressed without loss."""
    from gpu_util import run_step
    base = synth.LayerSpec("inv", 3, 8, 8, 12, 12, 3, 3, 1, 1, 1, dtype)
    t = synth.make_inputs(base, "inv")
    res = {k: run_step(base.with_k(k), t) for k in (1, 2, 4)}
    assert np.array_equal(res[1]["Z"], t["X"].astype(np.float64))           # bit-exact copy
    g = geom(base)
    exact = oracle.conv_dw(g, t["X"].astype(np.float64), t["dY"].astype(np.float64))
    assert rel_l2(res[1]["dW"], exact) <= (1e-5 if dtype == synth.F32 else TIGHT)
    for k in (2, 4):
        assert np.array_equal(res[k]["Y"], res[1]["Y"])
        assert np.array_equal(res[k]["dX"], res[1]["dX"])
        assert np.array_equal(res[k]["db"], res[1]["db"])
        assert not np.array_equal(res[k]["dW"], res[1]["dW"])
    for k in (2, 4):
        spec = base.with_k(k)
        tc = dict(t, X=tile_constant_activation(spec))
        lossy = run_step(spec, tc)
        ref = run_step(spec.with_k(1), tc)
        assert rel_l2(lossy["dW"], ref["dW"]) <= 1e-5
        # average pooling keeps every channel's sum (up to storage rounding of Z)
    spec = base.with_k(2)
    Zsum = res[2]["Z"].sum(axis=(2, 3)) * 4
    np.testing.assert_allclose(Zsum, t["X"].astype(np.float64).sum(axis=(2, 3)),
                               rtol=1e-5 if dtype == synth.F32 else 4e-3)


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_gradient_cosine(dtype):
    """Layer sensitivity metric: cosine of the weight gradient from the compressed activation
    against the exact one, computed on the device, against the oracle's."""
    import torch
    from gpu_util import run_step, upload, workspace, Guarded
    from paper_2409_11902_amd import binding as B
    spec = synth.LayerSpec("cos", 3, 24, 40, 14, 14, 3, 3, 1, 1, 2, dtype)
    t = synth.make_inputs(spec, "cos")
    lossy, exact = run_step(spec, t), run_step(spec.with_k(1), t)
    d = lossy["desc"]
    a, b = upload(lossy["dW"].astype(np.float32), synth.F32), upload(exact["dW"].astype(np.float32), synth.F32)
    out = Guarded((4,), torch.float32)
    for _ in range(2):  # twice: the workspace is reused, the result must not change
        B.cac_grad_cosine(d, a, b, out.t, workspace(d, B.OP_GRAD_COSINE))
    torch.cuda.synchronize()
    out.check("cosine")
    got = out.t.cpu().numpy().astype(np.float64)
    # (a) the reduction itself: against fp64 sums of the very same device gradients
    av, bv = lossy["dW"].ravel(), exact["dW"].ravel()
    np.testing.assert_allclose(got[1:], [av @ bv, av @ av, bv @ bv], rtol=2e-6)
    assert abs(got[0] - oracle.cosine(lossy["dW"], exact["dW"])) <= 2e-6
    # (b) the metric end to end: against the oracle's gradients from the oracle's pooled map
    g = geom(spec)
    X, dY = t["X"].astype(np.float64), t["dY"].astype(np.float64)
    xh = oracle.inflate(oracle.avgpool(X, 2, 2), spec.H, spec.W, 2, 2)
    want = oracle.cosine(oracle.conv_dw(g, xh, dY), oracle.conv_dw(g, X, dY))
    assert 0.3 < want < 0.999   # compression changes the direction, but not arbitrarily
    assert abs(got[0] - want) <= (1e-5 if dtype == synth.F32 else 2e-3)
    # degenerate input: a zero gradient has no direction
    B.cac_grad_cosine(d, a, torch.zeros_like(b), out.t, workspace(d, B.OP_GRAD_COSINE))
    torch.cuda.synchronize()
    assert out.t[0].item() == 0.0


def test_weight_gradient_is_reproducible_bit_for_bit():
    """The pixel slices are summed in a fixed order (no atomics): the same call twice, and the
    same call after unrelated work, gives identical bits."""
    from gpu_util import run_step
    for case in (("repro a", 9, 64, 64, 8, 8, 3, 3, 1, 1, 2), ("repro b", 6, 40, 72, 14, 14, 3, 3, 1, 1, 2),
                 ("repro c", 4, 64, 128, 14, 14, 1, 1, 2, 0, 2)):
        name, N, C, K, H, W, R, S, st, pad, k = case
        spec = synth.LayerSpec(name, N, C, K, H, W, R, S, st, pad, k, synth.BF16)
        t = synth.make_inputs(spec, "repro")
        first = run_step(spec, t)["dW"]
        run_step(spec.with_k(1), t)
        assert np.array_equal(first, run_step(spec, t)["dW"])


@pytest.mark.parametrize("shape", [(3, 24, 40, 16, 16), (2, 64, 64, 8, 32), (5, 70, 16, 4, 8), (7, 72, 16, 4, 4), (3, 20, 8, 6, 4)])
def test_pooling_fused_into_the_forward_pass_equals_the_standalone_kernel(shape):
    """Where the forward pass forms Z on its way (2 x 2 tiles, rows of 4 or a multiple of 8 pixels),
    the bits are those of cac_compress."""
    import torch
    from gpu_util import upload, workspace
    from paper_2409_11902_amd import binding as B
    N, C, K, H, W = shape
    spec = synth.LayerSpec("fusedpool", N, C, K, H, W, 3, 3, 1, 1, 2, synth.BF16)
    t = synth.make_inputs(spec, "fusedpool")
    d = B.desc_from_spec(spec)
    X, Wt, b = (upload(t[k], spec.dtype) for k in ("X", "W", "b"))
    Y = torch.empty((N, K, spec.P, spec.Q), dtype=torch.bfloat16, device="cuda:0")
    Z1 = torch.full((N, C, H // 2, W // 2), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    Z2 = torch.full_like(Z1, float("nan"))
    B.conv_fwd_and_compress(d, X, Wt, b, Y, Z1, workspace(d, B.OP_FWD_AND_COMPRESS))
    B.cac_compress(d, X, Z2)
    torch.cuda.synchronize()
    assert torch.equal(Z1.view(torch.int16), Z2.view(torch.int16))
    want = oracle.avgpool(t["X"].astype(np.float64), 2, 2)
    assert np.abs(Z2.float().cpu().numpy() - want).max() <= np.abs(want).max() * 2.0 ** -8


@pytest.mark.parametrize("combined", [False, True], ids=["separate backward calls", "combined backward call"])
def test_graph_capture_and_side_stream(combined):
    """The three calls enqueue on the caller's stream only and record no memset nodes: captured
    in a HIP graph on a side stream and replayed several times, with eager work and
    synchronisations in between, every replay reproduces the eager result."""
    import torch
    from gpu_util import upload, workspace
    from paper_2409_11902_amd import binding as B
    spec = synth.LayerSpec("graph", 6, 40, 72, 14, 14, 3, 3, 2, 1, 2, synth.BF16)   # stride 2: dX clears + 4 classes
    t = synth.make_inputs(spec, "graph")
    d = B.desc_from_spec(spec)
    hp, wp, _, _ = B.cac_pooled_shape(d)
    X, Wt, b, dY = (upload(t[k], spec.dtype) for k in ("X", "W", "b", "dY"))
    bf = torch.bfloat16
    Y = torch.empty((spec.N, spec.K, spec.P, spec.Q), dtype=bf, device="cuda:0")
    Z = torch.empty((spec.N, spec.C, hp, wp), dtype=bf, device="cuda:0")
    dW = torch.empty((spec.K, spec.C, 3, 3), dtype=torch.float32, device="cuda:0")
    dX = torch.empty((spec.N, spec.C, spec.H, spec.W), dtype=bf, device="cuda:0")
    ws = [workspace(d, op) for op in (B.OP_FWD_AND_COMPRESS, B.OP_BWD_WEIGHT_COMPRESSED, B.OP_BWD_DATA,
                                      B.OP_BWD_WEIGHT_AND_DATA)]

    def step(stream):
        B.conv_fwd_and_compress(d, X, Wt, b, Y, Z, ws[0], stream)
        if combined:
            B.conv_bwd_weight_and_data(d, Z, Wt, dY, dW, dX, ws[3], stream)
        else:
            B.conv_bwd_weight_compressed(d, Z, dY, dW, ws[1], stream)
            B.conv_bwd_data(d, Wt, dY, dX, ws[2], stream)

    outs = (Y, Z, dW, dX)
    step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(side)                                  # eager on the side stream
        side.synchronize()
        for o, w in zip(outs, want):
            assert torch.equal(o, w)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step(side)
    torch.cuda.synchronize()
    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))                   # eager work between replays
        for w in ws:
            if w is not None:
                w.random_(0, 255)                   # the workspace carries nothing between calls
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, w in zip(outs, want):
            assert torch.equal(o, w), f"replay {rep}"


def test_no_bias_and_empty_free_paths():
    from gpu_util import run_step
    spec = synth.LayerSpec("nobias", 2, 4, 6, 8, 8, 3, 3, 1, 1, 2, synth.F32)
    t = synth.make_inputs(spec, "nobias")
    got = run_step(spec, t, has_bias=False)
    _check_step(spec, t, got, has_bias=False)


def test_probe_kernels_run_and_the_copy_copies():
    """The benchmark's yardstick kernels: the copy stream reproduces its source bit for bit and
    leaves what lies beyond untouched; the read stream and the MFMA loop run to completion."""
    import torch
    from paper_2409_11902_amd import binding as B
    n = (1 << 20) + 4096
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.full((n + 64,), 7, dtype=torch.uint8, device="cuda:0")
    B.cac_probe(B.PROBE_COPY, src, dst, n)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and bool((dst[n:] == 7).all())
    out = torch.zeros(8192, dtype=torch.uint8, device="cuda:0")
    B.cac_probe(B.PROBE_READ, src, out, n)
    B.cac_probe(B.PROBE_MFMA, src, out, n, iters=4)
    B.cac_probe(B.PROBE_MFMA_16X16, src, out, n, iters=4)
    B.cac_probe(B.PROBE_MFMA_1WAVE, src, out, n, iters=4)
    torch.cuda.synchronize()
