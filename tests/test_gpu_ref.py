"""goq_ref_coefficients (REF mode, Eq. 3, on the device) against the CPU oracle.  Both sides work
in fp64; the device goes through the macro-block's Gram matrix (A^T A = [b1 b2]^T X_q^T X_q [b1 b2]),
the oracle evaluates Eq. 3 token by token, so the unrounded pairs differ by fp64 rounding only:
they are held to 1e-9 of the pair's norm, and the stored fp16 bits may differ by at most one unit
in the last place in at most 0.1 % of the entries (a value that sits on a rounding boundary)."""
import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _run(goq, q, w16, X, lam):
    torch = gu.torch_cuda()
    out, inn = w16.shape
    tokens = X.shape[0]
    gn = inn // 128
    ws = torch.empty(goq.ref_workspace_bytes(inn), dtype=torch.uint8, device="cuda")
    craw = torch.full((out, gn, 2), float("nan"), dtype=torch.float64, device="cuda")
    c1 = torch.full((out, gn), -1, dtype=torch.int16, device="cuda")
    c2 = torch.full((out, gn), -1, dtype=torch.int16, device="cuda")
    goq.ref_coefficients(q["bw"], tokens, out, inn, gu.to_dev(w16.view(np.uint16)), gu.to_dev(q["codes"]),
                         gu.to_dev(q["pattern"]), gu.to_dev(q["signs"]), gu.to_dev(X.view(np.uint16)), lam, ws, craw, c1, c2)
    torch.cuda.synchronize()
    return craw.cpu().numpy(), c1.cpu().numpy().view(np.uint16), c2.cpu().numpy().view(np.uint16)


def _compare(craw, c1, c2, ref, rc):
    scale = np.maximum(np.linalg.norm(rc, axis=2, keepdims=True), 1e-30)
    assert np.max(np.abs(craw - rc) / scale) <= 1e-9
    for got, want in ((c1, ref["c1"]), (c2, ref["c2"])):
        d = np.abs(got.astype(np.int32) - want.astype(np.int32))
        assert d.max() <= 1 and np.mean(d != 0) <= 1e-3, (int(d.max()), float(np.mean(d != 0)))


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 1, 128), (7, 3, 256), (50, 17, 384), (130, 70, 256), (333, 100, 1024)])
def test_ref_matches_oracle(oracle, bw, shape):
    import paper_2605_26092_amd as goq
    tokens, out, inn = shape
    print("ref bw=%d tokens=%d out=%d in=%d" % (bw, tokens, out, inn), flush=True)
    W = goq_inputs.weights(out, inn, config_id=51, tensor_id=bw)
    q = oracle.quantize_geo(bw, W, threads=8)
    X = goq_inputs.activations_a16(tokens, inn, config_id=51, tensor_id=100 + tokens, outlier_frac=0.01)
    ref, rc = oracle.ref_coefficients(q, W, X, lam=1e-4, threads=8)
    _compare(*_run(goq, q, W, X, 1e-4), ref, rc)


def test_ref_special_cases(oracle):
    """identity inputs with and without a ridge (the GEO coefficients), weights in the span of the
    bases (exact recovery), a single token (rank-one system, ridge only), an all-zero macro-block."""
    import paper_2605_26092_amd as goq
    bw, out, inn = 3, 40, 128
    W = goq_inputs.weights(out, inn, config_id=52, tensor_id=1)
    W[5] = 0
    q = oracle.quantize_geo(bw, W)
    eye = np.eye(128, dtype=np.float16)
    craw, c1, c2 = _run(goq, q, W, eye, 0.0)
    assert np.array_equal(c1, q["c1"]) and np.array_equal(c2, q["c2"])
    assert np.all(craw[5] == 0) and c1[5, 0] == 0 and c2[5, 0] == 0
    ref, rc = oracle.ref_coefficients(q, W, eye, lam=1e-4)
    _compare(*_run(goq, q, W, eye, 1e-4), ref, rc)
    X1 = goq_inputs.activations_a16(1, inn, config_id=52, tensor_id=101)
    ref, rc = oracle.ref_coefficients(q, W, X1, lam=1e-4)
    _compare(*_run(goq, q, W, X1, 1e-4), ref, rc)
    d = oracle.dequant(q, want=("b1", "b2"))
    Ws = (0.5 * d["b1"] - 0.25 * d["b2"]).astype(np.float16)
    X = goq_inputs.activations_a16(33, inn, config_id=52, tensor_id=102)
    craw, c1, c2 = _run(goq, q, Ws, X, 0.0)
    live = np.any(d["b1"] != 0, axis=1)
    assert np.allclose(craw[live, 0, 0], 0.5, rtol=1e-9) and np.allclose(craw[live, 0, 1], -0.25, rtol=1e-9)


def test_ref_config3_sampled(oracle):
    """LLaMA-2-7B q projection (4096 x 4096) with 512 calibration tokens: full run on the device,
    the oracle checks a seeded sample of 24 output channels over all macro-blocks."""
    import paper_2605_26092_amd as goq
    bw, tokens, out, inn = 3, 512, 4096, 4096
    W = goq_inputs.weights(out, inn, config_id=3, tensor_id=bw)
    q = oracle.quantize_geo(bw, W, threads=8)
    X = goq_inputs.activations_a16(tokens, inn, config_id=3, tensor_id=100, outlier_frac=0.01)
    craw, c1, c2 = _run(goq, q, W, X, 1e-4)
    rows = np.sort(goq_inputs.rng(3, 998).choice(out, size=24, replace=False))
    qs = {k: (v[rows] if isinstance(v, np.ndarray) else v) for k, v in q.items()}
    ref, rc = oracle.ref_coefficients(qs, W[rows], X, lam=1e-4, threads=8)
    _compare(craw[rows], c1[rows], c2[rows], ref, rc)
