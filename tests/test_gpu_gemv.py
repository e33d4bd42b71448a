"""goq_gemv / goq_gemv_batch against the CPU oracle, element by element, on seeded inputs.

Tolerances (A16, fp32 accumulation against the fp64 oracle): max relative error <= 1e-3 with
the denominator floored at 1 % of the output rms, and normalised backward error
|y - y^| / sum_k |x_k||W^_ik| <= 1e-3 (~5e-4 |y| when y is stored as fp16).  For fp32 outputs the
backward error is additionally held to 2e-6: the GEMV hands x to the matrix instruction as block
fixed point with 24 bits below each 32-activation block's maximum, products are exact, sums are
fp32.  A8: the slab partials are exact integers by construction; y is held to 1e-5
normalised error against the fp64 oracle.

The library has two batch-1 kernels (streaming and row-owner) and picks by size; the parity cases
run under each of them, forced through goq_gemv_select, and under the automatic choice."""
import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

TOL = 1e-3
KERNELS = ["AUTO", "STREAM", "ROWS"]


@pytest.fixture(autouse=True)
def _automatic_kernel_choice_after_each_test():
    yield
    import paper_2605_26092_amd as goq
    goq.gemv_select(goq.GEMV_AUTO)


def _select(goq, kernel):
    goq.gemv_select(getattr(goq, "GEMV_" + kernel))


def _quantize(oracle, bw, out, inn, cid):
    W = goq_inputs.weights(out, inn, config_id=cid, tensor_id=bw)
    return oracle.quantize_geo(bw, W, threads=8)


def _run_gemv(goq, q, x_np, act, ytype, sx_np=None):
    torch = gu.torch_cuda()
    out, inn = q["codes"].shape
    packed = gu.pack_layer(goq, q)
    x = gu.to_dev(x_np.reshape(-1))
    sx = gu.to_dev(sx_np) if sx_np is not None else None
    y = torch.full((out,), float("nan"), dtype=torch.float32 if ytype == goq.F32 else torch.float16, device="cuda")
    goq.gemv(q["bw"], act, out, inn, packed, x, sx, y, ytype)
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("ytype_name", ["F32", "F16"])
@pytest.mark.parametrize("shape", [(1, 128), (64, 128), (3, 256), (17, 384), (200, 512), (1100, 1024), (600, 4096),
                                   (150, 6400), (8300, 256), (40, 4224), (33, 8192)])
def test_gemv_a16_small(oracle, bw, ytype_name, shape):
    """(8300, 256) has more 16-row tiles than the automatic choice gives the row-owner kernel;
    6400 = 50 macro-blocks spans two of that kernel's staging windows, 4224 = 33 leaves a single
    macro-block for the second window, 8192 = 64 fills two windows exactly."""
    import paper_2605_26092_amd as goq
    out, inn = shape
    q = _quantize(oracle, bw, out, inn, 31)
    x = goq_inputs.activations_a16(1, inn, config_id=31, tensor_id=100 + out, outlier_frac=0.01)
    ref = oracle.gemm_a16(q, x, threads=8)[0]
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    for kernel in KERNELS:
        print("gemv a16 bw=%d %s out=%d in=%d kernel=%s" % (bw, ytype_name, out, inn, kernel), flush=True)
        _select(goq, kernel)
        y = _run_gemv(goq, q, x, goq.A16, getattr(goq, ytype_name))
        e1, e2 = gu.a16_errors(y, ref, x[0], what_abs)
        assert e1 <= TOL and e2 <= TOL, (kernel, e1, e2)
        if ytype_name == "F32":
            assert e2 <= 2e-6, (kernel, e2)


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 128), (64, 128), (17, 384), (200, 768), (1100, 1024), (150, 6400), (40, 4224)])
def test_gemv_a8(oracle, bw, shape):
    import paper_2605_26092_amd as goq
    out, inn = shape
    q = _quantize(oracle, bw, out, inn, 32)
    xq, sx = goq_inputs.activations_a8(1, inn, config_id=32, tensor_id=200 + out)
    ref, _ = oracle.gemm_a8(q, xq, sx, threads=8)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    scale = (np.abs(xq[0].astype(np.float64)) * float(sx[0])) @ what_abs.T
    for kernel in KERNELS:
        print("gemv a8 bw=%d out=%d in=%d kernel=%s" % (bw, out, inn, kernel), flush=True)
        _select(goq, kernel)
        y = _run_gemv(goq, q, xq, goq.A8, goq.F32, sx_np=sx)
        assert np.max(np.abs(y - ref[0]) / scale) <= 1e-5, kernel


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 128), (17, 384), (200, 768), (1100, 1024)])
def test_gemv_a4(oracle, bw, shape):
    """Packed 4-bit activations (the W3/A4 and W4/A4 operating points): the definition is the
    integer one of the int8 path on the unpacked values."""
    import paper_2605_26092_amd as goq
    out, inn = shape
    print("gemv a4 bw=%d out=%d in=%d" % (bw, out, inn), flush=True)
    q = _quantize(oracle, bw, out, inn, 34)
    xq, sx = goq_inputs.activations_int(1, inn, 4, config_id=34, tensor_id=200 + out)
    xq[0, :8] = [-8, 7, -7, 0, 1, -1, -8, 7]               # the full nibble range incl. -8
    ref, _ = oracle.gemm_a8(q, xq, sx, threads=8)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    scale = (np.abs(xq[0].astype(np.float64)) * float(sx[0])) @ what_abs.T
    for kernel in KERNELS:
        _select(goq, kernel)
        y = _run_gemv(goq, q, goq_inputs.pack_int4(xq), goq.A4, goq.F32, sx_np=sx)
        assert np.max(np.abs(y - ref[0]) / scale) <= 1e-5, kernel


@pytest.mark.parametrize("kernel", ["STREAM", "ROWS"])
def test_gemv_edge_cases(oracle, kernel):
    """all-zero codes, extreme fp16 activations, int8 saturation, single basis (c2 = 0)."""
    import paper_2605_26092_amd as goq
    _select(goq, kernel)
    q = goq_inputs.canonical_random(3, 130, 256, config_id=33)
    q["codes"][:64] = 3                                   # zero state everywhere in the first 64 rows
    q["c2"][64:100] = 0                                   # K = 1 rows
    q["codes"][100:] = 0                                  # all +1
    x = np.full((1, 256), 65504.0, np.float16)
    x[0, ::2] = -65504.0
    x[0, 5] = 6e-8                                        # subnormal
    ref = oracle.gemm_a16(q, x)[0]
    y = _run_gemv(goq, q, x, goq.A16, goq.F32)
    assert np.all(y[:64] == 0.0)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    e1, e2 = gu.a16_errors(y, ref, x[0], what_abs)
    assert e2 <= 2e-6, e2
    xq = np.full((1, 256), 127, np.int8)
    xq[0, 1::2] = -127
    sx = np.array([0.5], np.float32)
    ref8, _ = oracle.gemm_a8(q, xq, sx)
    y8 = _run_gemv(goq, q, xq, goq.A8, goq.F32, sx_np=sx)
    scale = (np.abs(xq[0].astype(np.float64)) * 0.5) @ what_abs.T
    assert np.max(np.abs(y8 - ref8[0]) / np.maximum(scale, 1e-30)) <= 1e-5
    q1 = dict(q)
    q1["codes"] = np.zeros_like(q["codes"])
    q1["c1"] = np.full_like(q["c1"], np.float16(1.0).view(np.uint16))
    q1["c2"] = np.zeros_like(q["c2"])
    xs = goq_inputs.activations_a16(1, 256, config_id=33)
    yr = _run_gemv(goq, q1, xs, goq.A16, goq.F32)
    assert np.allclose(yr, xs.astype(np.float64).sum(), rtol=1e-5)


@pytest.mark.parametrize("kernel", KERNELS)
def test_gemv_batch_matches_single_calls(oracle, kernel):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    _select(goq, kernel)
    shapes = [(256, 512), (1100, 512), (200, 1024)]
    probs, refs, ys = [], [], []
    keep = []
    for i, (out, inn) in enumerate(shapes):
        q = _quantize(oracle, 3, out, inn, 34 + i)
        x = goq_inputs.activations_a16(1, inn, config_id=34, tensor_id=i)
        refs.append(oracle.gemm_a16(q, x, threads=8)[0])
        packed = gu.pack_layer(goq, q)
        xd = gu.to_dev(x.reshape(-1))
        y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        keep += [packed, xd]
        ys.append(y)
        probs.append((out, inn, packed, xd, None, y, goq.F32))
    goq.gemv_batch(3, goq.A16, probs)
    torch.cuda.synchronize()
    for y, ref in zip(ys, refs):
        e1, _ = gu.a16_errors(y.cpu().numpy(), ref, None)
        assert e1 <= TOL, e1


@pytest.mark.parametrize("bw", [3, 4])
def test_gemv_config1_full_size(oracle, bw):
    """BASELINE config 1: 4096 x 4096, seed 0, batch 1, fp16 N(0,1) activations."""
    import paper_2605_26092_amd as goq
    print("gemv config1 bw=%d" % bw, flush=True)
    q = _quantize(oracle, bw, 4096, 4096, 0)
    x = goq_inputs.activations_a16(1, 4096, config_id=0, tensor_id=100)
    ref = oracle.gemm_a16(q, x, threads=8)[0]
    for kernel in KERNELS:                                 # the automatic choice here is ROWS
        _select(goq, kernel)
        for ytype in (goq.F32, goq.F16):
            y = _run_gemv(goq, q, x, goq.A16, ytype)
            e1, _ = gu.a16_errors(y, ref, None)
            assert e1 <= TOL, (kernel, ytype, e1)


def test_gemv_two_streams_in_flight_and_repeatable(oracle):
    """Launches on two streams share the library's scratch regions round-robin (at most 8 in flight):
    interleaved launches of two different layers, whose row groups are split over many workgroups,
    must all give the single-launch result, bit for bit (the combine order is fixed)."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    goq.gemv_select(goq.GEMV_STREAM)
    layers = []
    for i, (out, inn) in enumerate([(1500, 2048), (700, 4096)]):
        q = _quantize(oracle, 3, out, inn, 36 + i)
        x = goq_inputs.activations_a16(1, inn, config_id=36, tensor_id=i)
        packed = gu.pack_layer(goq, q)
        xd = gu.to_dev(x.reshape(-1))
        y0 = torch.zeros(out, dtype=torch.float32, device="cuda")
        goq.gemv(3, goq.A16, out, inn, packed, xd, None, y0, goq.F32)
        torch.cuda.synchronize()
        ref = oracle.gemm_a16(q, x, threads=8)[0]
        e1, _ = gu.a16_errors(y0.cpu().numpy(), ref, None)
        assert e1 <= TOL
        layers.append((out, inn, packed, xd, y0))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for rep in range(6):
        for s, (out, inn, packed, xd, y0) in zip(streams, layers):
            y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
            with torch.cuda.stream(s):
                goq.gemv(3, goq.A16, out, inn, packed, xd, None, y, goq.F32, stream=s)
            outs.append((y, y0))
        if rep % 3 == 2:
            torch.cuda.synchronize()          # never more than 8 launches in flight
    torch.cuda.synchronize()
    for y, y0 in outs:
        assert torch.equal(y, y0)


def _one_hot_coefficients(q, g, which):
    """c1 (which = 0) or c2 (which = 1) equal to 1 in macro-block g, every other coefficient 0."""
    q = dict(q)
    one = np.float16(1.0).view(np.uint16)
    c = [np.zeros_like(q["c1"]), np.zeros_like(q["c2"])]
    if g is None:
        c[which][:, :] = one
    else:
        c[which][:, g] = one
    q["c1"], q["c2"] = c
    return q


@pytest.mark.parametrize("kernel", ["STREAM", "ROWS"])
@pytest.mark.parametrize("bw,act_name", [(3, "A8"), (4, "A8"), (3, "A4"), (4, "A4")])
def test_gemv_integer_slab_sums_bit_exact(oracle, bw, act_name, kernel):
    """Integer activations (Sec. 3.5, Eq. 4): the slab sums P1, P2 are exact integers.  The GEMV has
    no partials output, so they are read through y: with s_x = 1, c1 = 1 in one macro-block and every
    other coefficient 0, y 2^(E-1) IS that macro-block's P1 (likewise c2 and P2); with c1 = 1
    everywhere it is the sum of the P1 of all macro-blocks (< 2^24, exact in fp32).  Compared with
    the oracle's int32 partials, equality.  The activations mix the extremes of the range with +-1
    inside one micro-block and across the four micro-blocks that share a block scale of the
    matrix instruction (b, b+1, b+4, b+5), besides random values."""
    import paper_2605_26092_amd as goq
    _select(goq, kernel)
    out, inn = 200, 1024
    gn = inn // 128
    top = 127 if act_name == "A8" else 7
    q0 = goq_inputs.canonical_random(bw, out, inn, config_id=37, tensor_id=bw)
    r = goq_inputs.rng(37, 500 + bw)
    xq = r.integers(-top, top + 1, size=(1, inn)).astype(np.int8)
    xq[0, 0:8] = [top, 1, -top, -1, 1, top, -1, -top]             # extremes and +-1 in one micro-block
    xq[0, 128:136] = top                                          # micro-block 0 of slab 1 at the top,
    for m in (1, 4, 5):                                           # its scale partners at +-1
        xq[0, 128 + 8 * m:128 + 8 * m + 8] = [1, -1, 1, -1, -1, 1, -1, 1]
    xq[0, 256:384] = -top                                         # a saturated slab
    xq[0, 384:512] = 0                                            # an all-zero slab
    if act_name == "A4":
        xq[0, 512:520] = -8                                       # the nibble range's extra value
    sx = np.array([1.0], np.float32)
    _, parts = oracle.gemm_a8(q0, xq, sx, threads=8, want_partials=True)   # [1, out, gn, 2] int32
    scale = float(1 << ((1 << (bw - 1)) - 1))                     # 2^(E-1): 8 (bw 3), 128 (bw 4)
    xdev = goq_inputs.pack_int4(xq) if act_name == "A4" else xq
    for which in (0, 1):
        for g in list(range(gn)) + [None]:
            q = _one_hot_coefficients(q0, g, which)
            y = _run_gemv(goq, q, xdev, getattr(goq, act_name), goq.F32, sx_np=sx)
            want = parts[0, :, :, which].sum(axis=1) if g is None else parts[0, :, g, which]
            assert np.abs(want).max() < (1 << 24)
            assert np.array_equal(y * scale, want.astype(np.float64)), (which, g)


def test_mfma_probe_matches_the_assumptions_of_the_gemv():
    """The exactness of the batch-1 path rests on two measured properties of the 8-bit-float matrix
    instruction (goq_mfma_probe): the depth of the grid on which 8 products are added, and which
    activations share a block scale.  A hardware, microcode or compiler change that moves either is
    caught here by name."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    report = torch.full((17,), -1, dtype=torch.int32, device="cuda")
    goq.mfma_probe(report)
    torch.cuda.synchronize()
    rep = report.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
    print("mfma probe: depth %d, masks %s" % (rep[0], [hex(v) for v in rep[1:]]), flush=True)
    assert rep[0] >= 10, "grid depth %d: 3-bit digits x powers of two down to 2^-7 need 10 places" % rep[0]
    assert rep[0] == 13, "the grid depth changed (was 13): re-derive the digit width"
    for Q in range(4):
        half = 0xFFFF << (16 * (Q // 2))
        want = [half if i // 2 == Q % 2 else 0 for i in range(4)]
        assert list(rep[1 + 4 * Q:5 + 4 * Q]) == want, (Q, [hex(v) for v in rep[1 + 4 * Q:5 + 4 * Q]])
