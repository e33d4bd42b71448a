"""BASELINE configs 2 and 5 at full size, in the launch configuration bench.py times.

Config 2: the seven LLaMA-2-7B block GEMVs as ONE goq_gemv_batch launch (W3 as in the config, and
W4), every output checked against the oracle.  Config 5: LLaMA-2-70B shapes (k: 1024 x 8192, down: 8192 x 28672) as GEMV
(all outputs) and as a 512-token GEMM (a seeded sample of token rows, all outputs)."""
import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-3


def _quantize(oracle, bw, out, inn, cid, tid):
    W = goq_inputs.weights(out, inn, config_id=cid, tensor_id=tid)
    return oracle.quantize_geo(bw, W, threads=16)


@pytest.mark.parametrize("bw", [3, 4])
def test_config2_block_gemv_batch(oracle, bw):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    probs, refs, ys, keep = [], [], [], []
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_7B_BLOCK):
        print("config2 bw=%d %s %dx%d" % (bw, name, out, inn), flush=True)
        q = _quantize(oracle, bw, out, inn, 2, idx)
        x = goq_inputs.activations_a16(1, inn, config_id=2, tensor_id=100 + idx, outlier_frac=0.01)
        refs.append(oracle.gemm_a16(q, x, threads=16)[0])
        packed = gu.pack_layer(goq, q)
        xd = gu.to_dev(x.reshape(-1))
        y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        keep += [packed, xd]
        ys.append(y)
        probs.append((out, inn, packed, xd, None, y, goq.F32))
        del q
    for rep in range(2):                       # a second launch must not accumulate onto the first
        goq.gemv_batch(bw, goq.A16, probs)
    torch.cuda.synchronize()
    for (name, _, _), y, ref in zip(goq_inputs.LLAMA2_7B_BLOCK, ys, refs):
        e1, _ = gu.a16_errors(y.cpu().numpy(), ref, None)
        assert e1 <= TOL, (name, e1)


@pytest.mark.parametrize("name,out,inn", [("k", 1024, 8192), ("down", 8192, 28672)])
def test_config5_70b_shapes(oracle, name, out, inn):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    print("config5 %s %dx%d" % (name, out, inn), flush=True)
    q = _quantize(oracle, 3, out, inn, 5, 0)
    packed = gu.pack_layer(goq, q)
    x = goq_inputs.activations_a16(1, inn, config_id=5, tensor_id=100, outlier_frac=0.01)
    ref = oracle.gemm_a16(q, x, threads=16)[0]
    for ytype, dt in ((goq.F32, torch.float32), (goq.F16, torch.float16)):
        y = torch.full((out,), float("nan"), dtype=dt, device="cuda")
        goq.gemv(3, goq.A16, out, inn, packed, gu.to_dev(x.reshape(-1)), None, y, ytype)
        torch.cuda.synchronize()
        e1, _ = gu.a16_errors(y.float().cpu().numpy(), ref, None)
        assert e1 <= TOL, (ytype, e1)
    tokens = 512
    X = goq_inputs.activations_a16(tokens, inn, config_id=5, tensor_id=101, outlier_frac=0.01)
    Y = torch.full((tokens, out), float("nan"), dtype=torch.float16, device="cuda")
    goq.gemm(3, goq.A16, tokens, out, inn, packed, gu.to_dev(X), None, Y, goq.F16)
    torch.cuda.synchronize()
    rows = np.sort(goq_inputs.rng(5, 999).choice(tokens, size=6, replace=False))
    refm = oracle.gemm_a16(q, X[rows], threads=16)
    ym = Y[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    e1, _ = gu.a16_errors(ym, refm, None)
    assert e1 <= TOL, e1
    assert not torch.isnan(Y.float()).any()
