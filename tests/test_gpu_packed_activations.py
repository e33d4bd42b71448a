"""Packed 6-bit and 3-bit activations (GOQ_A6: four per three bytes, GOQ_A3: eight per three
bytes): storage formats, so every entry point must return, bit for bit, what it returns for the
same integers handed over as int8 (GOQ_A8), and the exported int32 slab partials must equal the
oracle's."""
import ctypes

import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _automatic_kernel_choice_after_each_test():
    yield
    import paper_2605_26092_amd as goq
    goq.gemv_select(goq.GEMV_AUTO)


FORMATS = {"A6": (6, "pack_int6"), "A3": (3, "pack_int3")}


def test_pack_layouts():
    """element k in bits b k .. b k + b - 1 of the row as a little-endian bit string (no GPU needed,
    but kept beside its users)"""
    for name, (bits, packer) in FORMATS.items():
        top = (1 << (bits - 1)) - 1
        xq = np.array([[-top - 1, top, -1, 0, 1, -2, top - 1, -top]], dtype=np.int8)
        p = getattr(goq_inputs, packer)(xq)
        assert p.shape == (1, bits) and p.dtype == np.uint8
        word = int.from_bytes(p[0].tobytes(), "little")
        for k, v in enumerate(xq[0]):
            f = (word >> (bits * k)) & ((1 << bits) - 1)
            assert (f - (1 << bits) if f > top else f) == int(v), (name, k)


@pytest.mark.parametrize("fmt", ["A6", "A3"])
@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("tokens,out,inn", [(70, 200, 512), (300, 130, 1280)])
def test_gemm_packed_equals_a8_and_oracle_partials(oracle, fmt, bw, tokens, out, inn):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    bits, packer = FORMATS[fmt]
    top = (1 << (bits - 1)) - 1
    print("gemm %s bw=%d %dx%dx%d" % (fmt, bw, tokens, out, inn), flush=True)
    q = oracle.quantize_geo(bw, goq_inputs.weights(out, inn, config_id=81, tensor_id=bw), threads=8)
    packed = gu.pack_layer(goq, q)
    xq, sx = goq_inputs.activations_int(tokens, inn, bits, config_id=81, tensor_id=200)
    assert xq.min() >= -top - 1 and xq.max() <= top
    # extremes of the format in one token
    xq[0, :8] = [-top - 1, top, -top - 1, top, -1, 0, 1, -top]
    ref, pref = oracle.gemm_a8(q, xq, sx, threads=8, want_partials=True)
    res = {}
    for name, act, Xd in (("A8", goq.A8, gu.to_dev(xq)), (fmt, getattr(goq, fmt), gu.to_dev(getattr(goq_inputs, packer)(xq)))):
        Y = torch.full((tokens, out), float("nan"), dtype=torch.float32, device="cuda")
        P = torch.zeros((tokens, out, inn // 128, 2), dtype=torch.int32, device="cuda")
        goq.gemm(bw, act, tokens, out, inn, packed, Xd, gu.to_dev(sx), Y, goq.F32, partials=P)
        Y2 = torch.full((tokens, out), float("nan"), dtype=torch.float32, device="cuda")
        goq.gemm(bw, act, tokens, out, inn, packed, Xd, gu.to_dev(sx), Y2, goq.F32)
        torch.cuda.synchronize()
        assert torch.equal(Y, Y2), name
        res[name] = (Y, P)
    assert torch.equal(res[fmt][0], res["A8"][0])
    assert torch.equal(res[fmt][1], res["A8"][1])
    assert np.array_equal(res[fmt][1].cpu().numpy(), pref)
    y = res[fmt][0].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(y - ref)) / (np.max(np.abs(ref)) + 1e-30) <= 1e-5


@pytest.mark.parametrize("fmt", ["A6", "A3"])
@pytest.mark.parametrize("bw", [3, 4])
def test_gemv_packed_equals_a8(oracle, fmt, bw):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    bits, packer = FORMATS[fmt]
    act_packed = getattr(goq, fmt)
    shapes = [(700, 512), (64, 4096), (1100, 1024), (33, 2048), (1, 128)]
    probs8, probs6, ys8, ys6, refs, keep = [], [], [], [], [], []
    for i, (out, inn) in enumerate(shapes):
        q = oracle.quantize_geo(bw, goq_inputs.weights(out, inn, config_id=82, tensor_id=i), threads=8)
        packed = gu.pack_layer(goq, q)
        xq, sx = goq_inputs.activations_int(1, inn, bits, config_id=82, tensor_id=200 + i)
        refs.append(oracle.gemm_a8(q, xq, sx, threads=8)[0][0])
        x8, x6, sxd = gu.to_dev(xq.reshape(-1)), gu.to_dev(getattr(goq_inputs, packer)(xq).reshape(-1)), gu.to_dev(sx)
        y8 = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        y6 = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        keep += [packed, x8, x6, sxd]
        ys8.append(y8)
        ys6.append(y6)
        probs8.append((out, inn, packed, x8, sxd, y8, goq.F32))
        probs6.append((out, inn, packed, x6, sxd, y6, goq.F32))
    for kernel in (goq.GEMV_STREAM, goq.GEMV_ROWS):
        goq.gemv_select(kernel)
        for y in ys8 + ys6:
            y.fill_(float("nan"))
        goq.gemv_batch(bw, goq.A8, probs8)
        goq.gemv_batch(bw, act_packed, probs6)
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(ys8, ys6)):
            assert torch.equal(a, b), (kernel, k)
            yn = b.cpu().numpy().astype(np.float64)
            assert np.max(np.abs(yn - refs[k])) / (np.max(np.abs(refs[k])) + 1e-30) <= 1e-5, (kernel, k)
    # the stream entry point
    ws = torch.empty(goq.gemv_workspace_bytes() + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:][:goq.gemv_workspace_bytes()]
    goq.gemv_workspace_init(ws)
    goq.gemv_select(goq.GEMV_STREAM)
    goq.gemv_batch(bw, goq.A8, probs8)
    th, nbytes = goq.gemv_stream_table(bw, act_packed, probs6)
    raw = np.frombuffer((ctypes.c_ubyte * nbytes).from_address(ctypes.addressof(th)), dtype=np.uint8).copy()
    td = torch.from_numpy(raw).cuda()
    for y in ys6:
        y.fill_(float("nan"))
    goq.gemv_stream(th, td, ws)
    torch.cuda.synchronize()
    for k, (a, b) in enumerate(zip(ys8, ys6)):
        assert torch.equal(a, b), ("stream", k)
