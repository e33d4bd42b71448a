"""goq_gemm against the CPU oracle on seeded inputs.

A16: element by element within the A16 tolerance (see test_gpu_gemv.py).  A8: the int32 slab
partials P1, P2 are compared bit for bit; the fp32 output is held to 1e-5 normalised error.
At the BASELINE shapes the GPU runs the full problem and the oracle checks a seeded sample of
token rows (all outputs)."""
import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-3


def _quantize(oracle, bw, out, inn, cid):
    W = goq_inputs.weights(out, inn, config_id=cid, tensor_id=bw)
    return oracle.quantize_geo(bw, W, threads=8)


def _gemm(goq, q, X_np, act, ytype, sx_np=None, want_partials=False):
    torch = gu.torch_cuda()
    out, inn = q["codes"].shape
    tokens = X_np.shape[0]
    packed = gu.pack_layer(goq, q)
    X = gu.to_dev(X_np)
    sx = gu.to_dev(sx_np) if sx_np is not None else None
    Y = torch.full((tokens, out), float("nan"), dtype=torch.float32 if ytype == goq.F32 else torch.float16, device="cuda")
    parts = None
    if want_partials:
        parts = torch.full((tokens, out, inn // 128, 2), -7777, dtype=torch.int32, device="cuda")
    goq.gemm(q["bw"], act, tokens, out, inn, packed, X, sx, Y, ytype, partials=parts)
    torch.cuda.synchronize()
    return Y, parts


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 16, 128), (5, 64, 128), (17, 130, 384), (130, 200, 256), (200, 384, 1024),
                                   (257, 1100, 512)])
def test_gemm_a16_small(oracle, bw, shape):
    import paper_2605_26092_amd as goq
    tokens, out, inn = shape
    print("gemm a16 bw=%d tokens=%d out=%d in=%d" % (bw, tokens, out, inn), flush=True)
    q = _quantize(oracle, bw, out, inn, 41)
    X = goq_inputs.activations_a16(tokens, inn, config_id=41, tensor_id=100 + tokens, outlier_frac=0.01)
    ref = oracle.gemm_a16(q, X, threads=8)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    for ytype in (goq.F32, goq.F16):
        Y, _ = _gemm(goq, q, X, goq.A16, ytype)
        y = Y.float().cpu().numpy().astype(np.float64)
        e1, e2 = gu.a16_errors(y, ref, X, what_abs)
        assert e1 <= TOL and e2 <= TOL, (ytype, e1, e2)
        if ytype == goq.F32:
            assert e2 <= 2e-6, e2


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 16, 128), (5, 64, 128), (17, 130, 384), (197, 768, 768), (300, 200, 3072)])
def test_gemm_a8_bit_exact_partials(oracle, bw, shape):
    import paper_2605_26092_amd as goq
    tokens, out, inn = shape
    print("gemm a8 bw=%d tokens=%d out=%d in=%d" % (bw, tokens, out, inn), flush=True)
    q = _quantize(oracle, bw, out, inn, 42)
    Xq, sx = goq_inputs.activations_a8(tokens, inn, config_id=42, tensor_id=200 + tokens)
    ref, rparts = oracle.gemm_a8(q, Xq, sx, threads=8, want_partials=True)
    Y, parts = _gemm(goq, q, Xq, goq.A8, goq.F32, sx_np=sx, want_partials=True)
    assert np.array_equal(parts.cpu().numpy(), rparts)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    scale = (np.abs(Xq.astype(np.float64)) * sx[:, None].astype(np.float64)) @ what_abs.T
    y = Y.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(y - ref) / np.maximum(scale, 1e-30)) <= 1e-5
    # without the partials output the result is the same
    Y2, _ = _gemm(goq, q, Xq, goq.A8, goq.F32, sx_np=sx)
    assert np.array_equal(Y2.cpu().numpy(), Y.cpu().numpy())


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 16, 128), (17, 130, 384), (197, 768, 768), (300, 200, 1024)])
def test_gemm_a4_bit_exact_partials(oracle, bw, shape):
    """Packed 4-bit activations: int32 slab partials bit for bit against the oracle's integer
    definition on the unpacked values."""
    import paper_2605_26092_amd as goq
    tokens, out, inn = shape
    print("gemm a4 bw=%d tokens=%d out=%d in=%d" % (bw, tokens, out, inn), flush=True)
    q = _quantize(oracle, bw, out, inn, 45)
    Xq, sx = goq_inputs.activations_int(tokens, inn, 4, config_id=45, tensor_id=200 + tokens)
    Xq[0, :8] = [-8, 7, -7, 0, 1, -1, -8, 7]
    ref, rparts = oracle.gemm_a8(q, Xq, sx, threads=8, want_partials=True)
    Y, parts = _gemm(goq, q, goq_inputs.pack_int4(Xq), goq.A4, goq.F32, sx_np=sx, want_partials=True)
    assert np.array_equal(parts.cpu().numpy(), rparts)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    scale = (np.abs(Xq.astype(np.float64)) * sx[:, None].astype(np.float64)) @ what_abs.T
    y = Y.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(y - ref) / np.maximum(scale, 1e-30)) <= 1e-5


def test_gemm_edge_cases(oracle):
    import paper_2605_26092_amd as goq
    q = goq_inputs.canonical_random(3, 70, 256, config_id=43)
    q["codes"][:16] = 3                                   # all-zero rows
    q["c2"][16:40] = 0                                    # K = 1 rows
    X = np.full((33, 256), 65504.0, np.float16)
    X[:, ::2] = -65504.0
    X[7] = 0
    ref = oracle.gemm_a16(q, X)
    Y, _ = _gemm(goq, q, X, goq.A16, goq.F32)
    y = Y.cpu().numpy().astype(np.float64)
    assert np.all(y[:, :16] == 0) and np.all(y[7] == 0)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    _, e2 = gu.a16_errors(y, ref, X, what_abs)
    assert e2 <= 2e-6, e2
    Xq = np.full((20, 256), 127, np.int8)
    Xq[:, 1::2] = -127
    q["codes"][40:] = 0                                   # all +1: the int32 headroom case
    sx = np.full(20, 0.25, np.float32)
    ref8, rp = oracle.gemm_a8(q, Xq, sx, want_partials=True)
    Y8, parts = _gemm(goq, q, Xq, goq.A8, goq.F32, sx_np=sx, want_partials=True)
    assert np.array_equal(parts.cpu().numpy(), rp)
    # bw = 4: the +1 state is 128 in units of 2^-7 (no int8); +-127 activations on it and on the
    # smallest state (-2^-7) give the largest and the smallest slab sums
    q4 = goq_inputs.canonical_random(4, 70, 256, config_id=44)
    q4["codes"][:35] = 0                                  # all +1
    q4["codes"][35:] = 15                                 # all -2^-7
    ref4, rp4 = oracle.gemm_a8(q4, Xq, sx, want_partials=True)
    Y4, parts4 = _gemm(goq, q4, Xq, goq.A8, goq.F32, sx_np=sx, want_partials=True)
    assert np.array_equal(parts4.cpu().numpy(), rp4)
    Xq[:] = 127                                           # no cancellation: 128 * 127 * 128 per slab
    ref4, rp4 = oracle.gemm_a8(q4, Xq, sx, want_partials=True)
    Y4, parts4 = _gemm(goq, q4, Xq, goq.A8, goq.F32, sx_np=sx, want_partials=True)
    assert np.array_equal(parts4.cpu().numpy(), rp4)
    assert np.max(np.abs(Y4.cpu().numpy().astype(np.float64) - ref4)) <= 1e-5 * np.max(np.abs(ref4))


@pytest.mark.parametrize("bw,name,out,inn", [(3, "q", 4096, 4096), (4, "q", 4096, 4096), (3, "down", 4096, 11008)])
def test_gemm_config3_sampled(oracle, bw, name, out, inn):
    """BASELINE config 3 (2048-token prefill, LLaMA-2-7B shapes): full GPU run, the oracle checks
    a seeded sample of 12 token rows over all outputs."""
    import paper_2605_26092_amd as goq
    print("gemm config3 bw=%d %s" % (bw, name), flush=True)
    tokens = 2048
    q = _quantize(oracle, bw, out, inn, 3)
    X = goq_inputs.activations_a16(tokens, inn, config_id=3, tensor_id=100, outlier_frac=0.01)
    Y, _ = _gemm(goq, q, X, goq.A16, goq.F16)
    rows = np.sort(goq_inputs.rng(3, 999).choice(tokens, size=12, replace=False))
    ref = oracle.gemm_a16(q, X[rows], threads=8)
    y = Y[gu.torch_cuda().from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    e1, _ = gu.a16_errors(y, ref, None)
    assert e1 <= TOL, e1


@pytest.mark.parametrize("bw,act_name", [(3, "A8"), (3, "A4"), (4, "A8")])
def test_gemm_config4_sampled(oracle, bw, act_name):
    """BASELINE config 4 (ViT-B fc1, 197 x 64 tokens, W3/A8; also the W3/A4 and W4/A8 operating
    points at the same size): full GPU run with the partials output, bit-exact on a seeded sample
    of 32 token rows."""
    import paper_2605_26092_amd as goq
    tokens, out, inn = 197 * 64, 3072, 768
    print("gemm config4 bw=%d %s" % (bw, act_name), flush=True)
    q = _quantize(oracle, bw, out, inn, 4)
    if act_name == "A8":
        Xq, sx = goq_inputs.activations_a8(tokens, inn, config_id=4, tensor_id=200)
        Y, parts = _gemm(goq, q, Xq, goq.A8, goq.F32, sx_np=sx, want_partials=True)
    else:
        Xq, sx = goq_inputs.activations_int(tokens, inn, 4, config_id=4, tensor_id=200)
        Y, parts = _gemm(goq, q, goq_inputs.pack_int4(Xq), goq.A4, goq.F32, sx_np=sx, want_partials=True)
    rows = np.sort(goq_inputs.rng(4, 999).choice(tokens, size=32, replace=False))
    ref, rp = oracle.gemm_a8(q, Xq[rows], sx[rows], threads=8, want_partials=True)
    idx = gu.torch_cuda().from_numpy(rows).cuda()
    assert np.array_equal(parts[idx].cpu().numpy(), rp)
    y = Y[idx].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(y - ref)) <= 1e-5 * np.max(np.abs(ref))


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(5, 64, 128), (17, 130, 384), (200, 384, 1024), (257, 1100, 512)])
def test_gemm_folded_ablation(oracle, bw, shape):
    """goq_gemm_folded rounds every weight c1 b1 + c2 b2 to fp16 (relative 2^-11 = 4.9e-4) before
    the product: normalised backward error <= 1e-3 against the oracle, and it agrees with goq_gemm
    to the same bound."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    tokens, out, inn = shape
    print("gemm folded bw=%d tokens=%d out=%d in=%d" % (bw, tokens, out, inn), flush=True)
    q = _quantize(oracle, bw, out, inn, 46)
    X = goq_inputs.activations_a16(tokens, inn, config_id=46, tensor_id=100 + tokens, outlier_frac=0.01)
    ref = oracle.gemm_a16(q, X, threads=8)
    what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
    packed = gu.pack_layer(goq, q)
    Xd = gu.to_dev(X)
    Y = torch.full((tokens, out), float("nan"), dtype=torch.float32, device="cuda")
    goq.gemm_folded(bw, tokens, out, inn, packed, Xd, Y, goq.F32)
    torch.cuda.synchronize()
    y = Y.cpu().numpy().astype(np.float64)
    _, e2 = gu.a16_errors(y, ref, X, what_abs)
    assert e2 <= TOL, e2
    Y2, _ = _gemm(goq, q, X, goq.A16, goq.F32)
    _, d2 = gu.a16_errors(y, Y2.cpu().numpy().astype(np.float64), X, what_abs)
    assert d2 <= TOL, d2


@pytest.mark.parametrize("bw,act_name", [(3, "A16"), (4, "A16"), (3, "A8"), (4, "A8")])
def test_gemm_batch_equals_single_calls(oracle, bw, act_name):
    """goq_gemm_batch: the tiles of several layers in one grid; bit for bit the results of the
    single calls (which are checked against the oracle above), partials included where asked."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    act = getattr(goq, act_name)
    shapes = [(70, 200, 256), (130, 64, 512), (33, 1100, 128)]
    probs, singles, keep = [], [], []
    for i, (tokens, out, inn) in enumerate(shapes):
        q = goq_inputs.canonical_random(bw, out, inn, config_id=47, tensor_id=i)
        packed = gu.pack_layer(goq, q)
        if act == goq.A16:
            X = gu.to_dev(goq_inputs.activations_a16(tokens, inn, config_id=47, tensor_id=10 + i))
            sx = None
        else:
            Xq, sxn = goq_inputs.activations_a8(tokens, inn, config_id=47, tensor_id=10 + i)
            X, sx = gu.to_dev(Xq), gu.to_dev(sxn)
        want_parts = act != goq.A16 and i != 1                 # a mix of problems with and without
        Y1 = torch.full((tokens, out), float("nan"), dtype=torch.float32, device="cuda")
        P1 = torch.full((tokens, out, inn // 128, 2), -7, dtype=torch.int32, device="cuda") if want_parts else None
        goq.gemm(bw, act, tokens, out, inn, packed, X, sx, Y1, goq.F32, partials=P1)
        Yb = torch.full((tokens, out), float("nan"), dtype=torch.float32, device="cuda")
        Pb = torch.full((tokens, out, inn // 128, 2), -7, dtype=torch.int32, device="cuda") if want_parts else None
        probs.append((tokens, out, inn, packed, X, sx, Yb, goq.F32, Pb))
        singles.append((Y1, P1, Yb, Pb))
        keep += [packed, X, sx]
    goq.gemm_batch(bw, act, probs)
    torch.cuda.synchronize()
    for Y1, P1, Yb, Pb in singles:
        assert torch.equal(Y1, Yb)
        if P1 is not None:
            assert torch.equal(P1, Pb)
