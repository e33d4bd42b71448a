"""Rows of the packed layout beyond `out` (the last 64-row block is padded) must not influence any
output: the padding is overwritten with random bytes after packing and every entry point must
return the same bits as with the padding goq_pack wrote."""
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


def _poison_padding(packed, bw, out, inn, seed):
    """random bytes into the quads (R = last row block, row >= out % 64) of every macro-block and chunk"""
    torch = gu.torch_cuda()
    ch = 4 if bw == 3 else 5
    gn = inn // 128
    R = (out + 63) // 64 - 1
    first = out - 64 * R                              # first padding row of the last block
    assert 0 < first < 64
    host = packed.cpu().numpy().copy()
    rng = np.random.default_rng(seed)
    for g in range(gn):
        for h in range(ch):
            base = (((R * gn + g) * ch + h) * 64) * 16       # byte offset of row 0's quad
            host[base + first * 16: base + 64 * 16] = rng.integers(0, 256, (64 - first) * 16, dtype=np.uint8)
    return torch.from_numpy(host).cuda()


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("out,inn", [(100, 512), (577, 1024)])
def test_padding_rows_do_not_reach_any_output(oracle, bw, out, inn):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    print("padding bw=%d %dx%d" % (bw, out, inn), flush=True)
    q = oracle.quantize_geo(bw, goq_inputs.weights(out, inn, config_id=71, tensor_id=bw), threads=8)
    clean = gu.pack_layer(goq, q)
    dirty = _poison_padding(clean, bw, out, inn, seed=bw * 1000 + out)
    assert not torch.equal(clean, dirty)

    # batch 1, both kernels, fp16 and int8 activations
    x = goq_inputs.activations_a16(1, inn, config_id=71, tensor_id=100, outlier_frac=0.01)
    xq, sx = goq_inputs.activations_int(1, inn, 8, config_id=71, tensor_id=200)
    for kernel in (goq.GEMV_STREAM, goq.GEMV_ROWS):
        goq.gemv_select(kernel)
        for act, xd, sxd in ((goq.A16, gu.to_dev(x.reshape(-1)), None), (goq.A8, gu.to_dev(xq.reshape(-1)), gu.to_dev(sx))):
            ys = []
            for pk in (clean, dirty):
                y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
                goq.gemv(bw, act, out, inn, pk, xd, sxd, y, goq.F32)
                torch.cuda.synchronize()
                ys.append(y)
            assert torch.equal(ys[0], ys[1]), (kernel, act)
            assert not torch.isnan(ys[0]).any()

    # many tokens (ragged token count), fp16 and int8 activations
    T = 70
    X = goq_inputs.activations_a16(T, inn, config_id=71, tensor_id=101, outlier_frac=0.01)
    Xq, sX = goq_inputs.activations_int(T, inn, 8, config_id=71, tensor_id=201)
    for act, Xd, sXd in ((goq.A16, gu.to_dev(X), None), (goq.A8, gu.to_dev(Xq), gu.to_dev(sX))):
        Ys = []
        for pk in (clean, dirty):
            Y = torch.full((T, out), float("nan"), dtype=torch.float32, device="cuda")
            goq.gemm(bw, act, T, out, inn, pk, Xd, sXd, Y, goq.F32)
            torch.cuda.synchronize()
            Ys.append(Y)
        assert torch.equal(Ys[0], Ys[1]), act
        assert not torch.isnan(Ys[0]).any()

    # unpack returns the canonical arrays of the real rows whatever the padding holds
    outs = []
    for pk in (clean, dirty):
        codes = torch.empty((out, inn), dtype=torch.uint8, device="cuda")
        pat = torch.empty((out, inn // 8), dtype=torch.uint8, device="cuda")
        sg = torch.empty((out, inn // 8), dtype=torch.uint8, device="cuda")
        c1 = torch.empty((out, inn // 128), dtype=torch.int16, device="cuda")
        c2 = torch.empty((out, inn // 128), dtype=torch.int16, device="cuda")
        goq.unpack(bw, out, inn, pk, codes, pat, sg, c1, c2)
        torch.cuda.synchronize()
        outs.append((codes, pat, sg, c1, c2))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert np.array_equal(outs[1][0].cpu().numpy(), q["codes"])
