"""goq_gemv_stream (a whole stream of batch-1 layers in one launch, problem table in device memory)
and goq_gemv_batch_ws (caller-owned workspace) against the CPU oracle and against goq_gemv_batch.

Tolerances as in test_gpu_gemv.py: A16 max relative error <= 1e-3 (denominator floored at 1 % of
the output rms) and, for fp32 outputs, normalised backward error <= 2e-6; integer activations
<= 1e-5 normalised.  Where two entry points run the same decomposition the results must be equal
bit for bit."""
import ctypes

import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(autouse=True)
def _automatic_kernel_choice_after_each_test():
    yield
    import paper_2605_26092_amd as goq
    goq.gemv_select(goq.GEMV_AUTO)


def _workspace(goq):
    torch = gu.torch_cuda()
    ws = torch.empty(goq.gemv_workspace_bytes() + 256, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + goq.gemv_workspace_bytes()]
    ws.fill_(0x5A)                                  # poisoned: workspace_init must clear what matters
    goq.gemv_workspace_init(ws)
    return ws


def _table_to_device(table_host, nbytes):
    torch = gu.torch_cuda()
    raw = np.frombuffer((ctypes.c_ubyte * nbytes).from_address(ctypes.addressof(table_host)), dtype=np.uint8).copy()
    return torch.from_numpy(raw).cuda()


def _problems(goq, oracle, bw, act_name, shapes, cid):
    """Quantise, pack and upload one problem per shape; returns (problem tuples, outputs, oracle refs,
    backward-error scales, keep-alive list)."""
    torch = gu.torch_cuda()
    probs, ys, refs, scales, keep = [], [], [], [], []
    for i, (out, inn) in enumerate(shapes):
        W = goq_inputs.weights(out, inn, config_id=cid, tensor_id=i)
        q = oracle.quantize_geo(bw, W, threads=8)
        packed = gu.pack_layer(goq, q)
        what_abs = np.abs(oracle.dequant(q, want=("what",))["what"])
        if act_name == "A16":
            x = goq_inputs.activations_a16(1, inn, config_id=cid, tensor_id=100 + i, outlier_frac=0.01)
            refs.append(oracle.gemm_a16(q, x, threads=8)[0])
            scales.append(np.abs(x[0].astype(np.float64)) @ what_abs.T)
            xd, sxd = gu.to_dev(x.reshape(-1)), None
        else:
            bits = 8 if act_name == "A8" else 4
            xq, sx = goq_inputs.activations_int(1, inn, bits, config_id=cid, tensor_id=200 + i)
            ref, _ = oracle.gemm_a8(q, xq, sx, threads=8)
            refs.append(ref[0])
            scales.append((np.abs(xq[0].astype(np.float64)) * float(sx[0])) @ what_abs.T)
            xd = gu.to_dev((goq_inputs.pack_int4(xq) if bits == 4 else xq).reshape(-1))
            sxd = gu.to_dev(sx)
        y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        keep += [packed, xd, sxd]
        ys.append(y)
        probs.append((out, inn, packed, xd, sxd, y, goq.F32))
    return probs, ys, refs, scales, keep


def _check(ys, refs, scales, act_name):
    for k, (y, ref, scale) in enumerate(zip(ys, refs, scales)):
        yn = y.cpu().numpy().astype(np.float64)
        assert not np.isnan(yn).any(), k
        e2 = np.max(np.abs(yn - ref) / np.maximum(scale, 1e-300))
        if act_name == "A16":
            e1, _ = gu.a16_errors(yn, ref, None)
            assert e1 <= TOL and e2 <= 2e-6, (k, e1, e2)
        else:
            assert e2 <= 1e-5, (k, e2)


# ragged outputs, one-slab and many-slab rows, a layer smaller than a row group, one that a piece
# boundary cuts several times, 20 problems so that pieces span several problems
SHAPES = [(1, 128), (700, 512), (64, 4096), (1100, 1024), (33, 2048), (513, 256), (200, 768), (3000, 128),
          (150, 6400), (17, 384)] * 2


@pytest.mark.parametrize("bw,act_name", [(3, "A16"), (4, "A16"), (3, "A8"), (4, "A8"), (3, "A4"), (4, "A4")])
def test_stream_small_problems_against_oracle(oracle, bw, act_name):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    print("gemv stream bw=%d %s, %d problems" % (bw, act_name, len(SHAPES)), flush=True)
    probs, ys, refs, scales, keep = _problems(goq, oracle, bw, act_name, SHAPES, 61)
    ws = _workspace(goq)
    th, nbytes = goq.gemv_stream_table(bw, getattr(goq, act_name), probs)
    td = _table_to_device(th, nbytes)
    goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    _check(ys, refs, scales, act_name)
    # a second launch on the same workspace: same bits (fixed combine order, counters back at zero)
    first = [y.clone() for y in ys]
    for y in ys:
        y.fill_(float("nan"))
    goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    for a, b in zip(first, ys):
        assert torch.equal(a, b)


@pytest.mark.parametrize("bw", [3, 4])
def test_stream_of_one_batch_equals_batch_and_batch_ws(oracle, bw):
    """The same problems through goq_gemv_batch (library scratch, streaming kernel forced),
    goq_gemv_batch_ws (caller workspace) and goq_gemv_stream run the same decomposition: equal
    bits."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    shapes = [(1500, 2048), (700, 4096), (4096, 512), (130, 128), (2050, 1024)]
    probs, ys, refs, scales, keep = _problems(goq, oracle, bw, "A16", shapes, 62)
    goq.gemv_select(goq.GEMV_STREAM)
    goq.gemv_batch(bw, goq.A16, probs)
    torch.cuda.synchronize()
    _check(ys, refs, scales, "A16")
    base = [y.clone() for y in ys]
    ws = _workspace(goq)
    for rep in range(2):
        for y in ys:
            y.fill_(float("nan"))
        goq.gemv_batch_ws(bw, goq.A16, probs, ws)
        torch.cuda.synchronize()
        for a, b in zip(base, ys):
            assert torch.equal(a, b), "goq_gemv_batch_ws, launch %d" % rep
    for y in ys:
        y.fill_(float("nan"))
    th, nbytes = goq.gemv_stream_table(bw, goq.A16, probs)
    td = _table_to_device(th, nbytes)
    goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    for a, b in zip(base, ys):
        assert torch.equal(a, b), "goq_gemv_stream"


def test_more_streams_than_static_regions(oracle):
    """goq_gemv on 12 different streams, one after the other (each stream idle before the next
    launches): the library's 8 static regions are taken over from idle streams, results stay
    bit-identical; then all 12 again, interleaved, with synchronisation every 8 launches."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    goq.gemv_select(goq.GEMV_STREAM)
    out, inn = 1500, 2048
    q = oracle.quantize_geo(3, goq_inputs.weights(out, inn, config_id=63, tensor_id=0), threads=8)
    x = goq_inputs.activations_a16(1, inn, config_id=63, tensor_id=100)
    packed = gu.pack_layer(goq, q)
    xd = gu.to_dev(x.reshape(-1))
    y0 = torch.zeros(out, dtype=torch.float32, device="cuda")
    goq.gemv(3, goq.A16, out, inn, packed, xd, None, y0, goq.F32)
    torch.cuda.synchronize()
    e1, _ = gu.a16_errors(y0.cpu().numpy(), oracle.gemm_a16(q, x, threads=8)[0], None)
    assert e1 <= TOL
    streams = [torch.cuda.Stream() for _ in range(12)]
    for rnd in range(2):
        outs = []
        for i, s in enumerate(streams):
            y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
            goq.gemv(3, goq.A16, out, inn, packed, xd, None, y, goq.F32, stream=s)
            outs.append(y)
            if rnd == 0 or i % 8 == 7:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        for y in outs:
            assert torch.equal(y, y0)


def test_config2_stream_of_32_blocks_full_size(oracle):
    """BASELINE config 2 in the launch configuration bench.py times: the seven W3/A16 GEMVs of a
    LLaMA-2-7B decoder block, 32 blocks (one token through a 32-block model's projections) as ONE
    goq_gemv_stream launch; every block has activations of its own, every output of every block
    is checked against the oracle."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    nblocks = 32
    packed, canon = [], []
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_7B_BLOCK):
        print("config2 stream: quantise %s %dx%d" % (name, out, inn), flush=True)
        q = oracle.quantize_geo(3, goq_inputs.weights(out, inn, config_id=2, tensor_id=idx), threads=16)
        packed.append(gu.pack_layer(goq, q))
        canon.append(q)
    probs, ys, xs = [], [], []
    for b in range(nblocks):
        for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_7B_BLOCK):
            x = goq_inputs.activations_a16(1, inn, config_id=2, tensor_id=1000 + 7 * b + idx, outlier_frac=0.01)
            xd = gu.to_dev(x.reshape(-1))
            y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
            xs.append((x, xd))
            ys.append(y)
            probs.append((out, inn, packed[idx], xd, None, y, goq.F32))
    ws = _workspace(goq)
    th, nbytes = goq.gemv_stream_table(3, goq.A16, probs)
    td = _table_to_device(th, nbytes)
    print("config2 stream: launch, %d problems" % len(probs), flush=True)
    for rep in range(2):
        goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    worst = 0.0
    for k, y in enumerate(ys):
        ref = oracle.gemm_a16(canon[k % 7], xs[k][0], threads=16)[0]
        e1, _ = gu.a16_errors(y.cpu().numpy(), ref, None)
        worst = max(worst, e1)
        assert e1 <= TOL, (k // 7, goq_inputs.LLAMA2_7B_BLOCK[k % 7][0], e1)
    print("config2 stream: worst relative error %.3g" % worst, flush=True)


@pytest.mark.parametrize("bw,act_name", [(3, "A16"), (4, "A8")])
def test_stream_of_thousands_of_tiny_problems(oracle, bw, act_name):
    """3000 problems of one to three units each (five small layers reused with activations of their
    own): every piece of the launch spans several problems, windows of staged activations cross
    many problem boundaries, most row groups end inside a window."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    layers = [(1, 128), (64, 128), (70, 256), (130, 128), (33, 384)]
    base = []
    for i, (out, inn) in enumerate(layers):
        q = oracle.quantize_geo(bw, goq_inputs.weights(out, inn, config_id=64, tensor_id=i), threads=8)
        base.append((q, gu.pack_layer(goq, q)))
    rng = np.random.default_rng(640 + bw)
    nprob = 3000
    pick = rng.integers(0, len(layers), nprob)
    probs, ys, refs, keep = [], [], [], []
    for k in range(nprob):
        q, packed = base[pick[k]]
        out, inn = layers[pick[k]]
        if act_name == "A16":
            x = goq_inputs.activations_a16(1, inn, config_id=64, tensor_id=1000 + k, outlier_frac=0.01)
            refs.append(oracle.gemm_a16(q, x, threads=1)[0])
            xd, sxd = gu.to_dev(x.reshape(-1)), None
        else:
            xq, sx = goq_inputs.activations_int(1, inn, 8, config_id=64, tensor_id=1000 + k)
            refs.append(oracle.gemm_a8(q, xq, sx, threads=1)[0][0])
            xd, sxd = gu.to_dev(xq.reshape(-1)), gu.to_dev(sx)
        y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        keep += [xd, sxd]
        ys.append(y)
        probs.append((out, inn, packed, xd, sxd, y, goq.F32))
    print("tiny-problem stream: %d problems, bw=%d %s" % (nprob, bw, act_name), flush=True)
    ws = _workspace(goq)
    th, nbytes = goq.gemv_stream_table(bw, getattr(goq, act_name), probs)
    td = _table_to_device(th, nbytes)
    for rep in range(2):
        goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    worst = 0.0
    for k in range(nprob):
        yn = ys[k].cpu().numpy().astype(np.float64)
        assert not np.isnan(yn).any(), k
        ref = refs[k]
        e = float(np.max(np.abs(yn - ref) / np.maximum(np.abs(ref), 1e-2 * np.sqrt(np.mean(ref ** 2)) + 1e-30)))
        worst = max(worst, e)
        assert e <= TOL, (k, layers[pick[k]], e)
    print("tiny-problem stream: worst relative error %.3g" % worst, flush=True)


def test_stream_with_the_maximum_number_of_problems(oracle):
    """GOQ_MAX_STREAM = 65536 problems in one table (one more is refused on the host): the same
    70 x 256 layer and activations 65536 times, each problem writing its own slice of one output
    buffer; every slice must equal the first bit for bit and the oracle within tolerance."""
    import paper_2605_26092_amd as goq
    from paper_2605_26092_amd import binding
    torch = gu.torch_cuda()
    out, inn, n = 70, 256, 65536
    q = oracle.quantize_geo(3, goq_inputs.weights(out, inn, config_id=65, tensor_id=0), threads=8)
    x = goq_inputs.activations_a16(1, inn, config_id=65, tensor_id=100, outlier_frac=0.01)
    ref = oracle.gemm_a16(q, x, threads=8)[0]
    packed, xd = gu.pack_layer(goq, q), gu.to_dev(x.reshape(-1))
    pitch = 80                                                     # floats per slice: 16-byte aligned slices
    ybuf = torch.full((n * pitch,), float("nan"), dtype=torch.float32, device="cuda")
    arr = (binding._Desc * n)()
    base = ybuf.data_ptr()
    for i in range(n):
        d = arr[i]
        d.out, d.in_, d.packed, d.x, d.sx, d.y, d.ytype = out, inn, packed.data_ptr(), xd.data_ptr(), None, base + 4 * pitch * i, goq.F32
    nbytes = ctypes.c_size_t(0)
    L = goq.lib()
    assert L.goq_gemv_stream_table_bytes(n + 1, ctypes.byref(nbytes)) == binding.ESHAPE
    print("max-size stream: %d problems" % n, flush=True)
    ws = _workspace(goq)
    th, tbytes = goq.gemv_stream_table(3, goq.A16, arr)
    td = _table_to_device(th, tbytes)
    goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    y = ybuf.view(n, pitch)[:, :out]
    assert not torch.isnan(y).any()
    assert torch.equal(y, y[0:1].expand(n, out))
    e1, _ = gu.a16_errors(y[0].cpu().numpy(), ref, None)
    assert e1 <= TOL, e1
    assert torch.isnan(ybuf.view(n, pitch)[:, out:]).all()         # nothing written past a slice's rows
