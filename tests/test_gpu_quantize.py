"""goq_quantize (GEO mode on the device) against the CPU oracle's quantizer: codes, pattern, signs
and the fp16 bits of c1, c2 must be IDENTICAL -- both sides work in fp64 with sums in ascending k,
every product has a power-of-two factor (exact), so there is one rounding sequence.  Where a cross
term is exactly zero the paper allows either sign; both sides take +1, so the bits still agree."""
import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _run(goq, bw, w16):
    torch = gu.torch_cuda()
    out, inn = w16.shape
    wd = gu.to_dev(w16.view(np.uint16))
    codes = torch.full((out, inn), 255, dtype=torch.uint8, device="cuda")
    pat = torch.full((out, inn // 8), 255, dtype=torch.uint8, device="cuda")
    sg = torch.full((out, inn // 8), 255, dtype=torch.uint8, device="cuda")
    c1 = torch.full((out, inn // 128), -1, dtype=torch.int16, device="cuda")
    c2 = torch.full((out, inn // 128), -1, dtype=torch.int16, device="cuda")
    goq.quantize(bw, out, inn, wd, codes, pat, sg, c1, c2)
    torch.cuda.synchronize()
    return {"codes": codes.cpu().numpy(), "pattern": pat.cpu().numpy(), "signs": sg.cpu().numpy(),
            "c1": c1.cpu().numpy().view(np.uint16), "c2": c2.cpu().numpy().view(np.uint16)}


def _same(got, ref):
    for k in ("codes", "pattern", "signs", "c1", "c2"):
        assert np.array_equal(got[k], ref[k]), (k, int(np.sum(got[k] != ref[k])))


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 128), (3, 256), (17, 384), (64, 128), (200, 512), (1100, 1024)])
def test_quantize_matches_oracle(oracle, bw, shape):
    import paper_2605_26092_amd as goq
    out, inn = shape
    print("quantize bw=%d out=%d in=%d" % (bw, out, inn), flush=True)
    w = goq_inputs.weights(out, inn, config_id=41, tensor_id=out + bw)
    _same(_run(goq, bw, w), oracle.quantize_geo(bw, w, threads=8))


@pytest.mark.parametrize("bw", [3, 4])
def test_quantize_degenerate_blocks(oracle, bw):
    """all-zero macro-block, all-equal weights, exact rounding ties, a single nonzero, subnormals,
    the largest finite fp16, and cross terms that are exactly zero."""
    import paper_2605_26092_amd as goq
    r = np.random.default_rng(5)
    rows = []
    rows.append(np.zeros(128))                                         # all zero
    rows.append(np.full(128, 0.37))                                    # all equal
    ties = np.tile(np.array([1.0, 0.75, 0.375, 0.1875, 0.125, -0.0625, -0.1875, -0.75]), 16)
    rows.append(ties)                                                  # midpoints of the 3-bit lattice
    one = np.zeros(128); one[77] = -0.5
    rows.append(one)                                                   # single nonzero
    rows.append(r.normal(0, 1e-6, 128))                                # fp16 subnormals
    big = r.normal(0, 1.0, 128); big[5] = 65504.0
    rows.append(big)
    rows.append(np.tile(np.array([1.0, 1.0, -1.0, -1.0, 0.5, 0.5, -0.5, -0.5]), 16))   # zero cross terms
    rows.append(r.choice([1.0, 0.5, 0.25, 0.125, 0.0, -1.0, -0.5], size=128))           # exactly representable
    w = np.stack(rows).astype(np.float16)
    _same(_run(goq, bw, w), oracle.quantize_geo(bw, w, threads=1))


def test_quantize_llama_shape_and_pack_gemv(oracle):
    """A full-width matrix (in = 4096, the width of BASELINE config 1) quantized on the device
    feeds goq_pack and goq_gemv directly; compared with the oracle end to end."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    out, inn = 512, 4096
    w = goq_inputs.weights(out, inn, config_id=0, tensor_id=3)
    ref = oracle.quantize_geo(3, w, threads=8)
    got = _run(goq, 3, w)
    _same(got, ref)
    got["bw"] = 3
    packed = gu.pack_layer(goq, got)
    x = goq_inputs.activations_a16(1, inn, config_id=0, tensor_id=100)
    y = torch.zeros(out, dtype=torch.float32, device="cuda")
    goq.gemv(3, goq.A16, out, inn, packed, gu.to_dev(x.reshape(-1)), None, y, goq.F32)
    torch.cuda.synchronize()
    yref = oracle.gemm_a16(ref, x, threads=8)[0]
    e1, _ = gu.a16_errors(y.cpu().numpy(), yref, None)
    assert e1 <= 1e-3, e1
