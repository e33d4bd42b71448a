"""goq_gemv_batch, the entry point that allocates nothing, recorded into a HIP graph (what a caller
under stream capture does) and replayed: every replay must reproduce the eager result bit for bit,
with the program's own eager work and synchronisations between the replays."""
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


@pytest.mark.parametrize("kernel_name", ["GEMV_STREAM", "GEMV_ROWS"])
def test_gemv_batch_replayed_from_a_graph(oracle, kernel_name):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    goq.gemv_select(getattr(goq, kernel_name))
    shapes = [(1500, 2048), (700, 4096), (130, 512)]
    probs, ys, refs, keep = [], [], [], []
    for i, (out, inn) in enumerate(shapes):
        q = oracle.quantize_geo(3, goq_inputs.weights(out, inn, config_id=83, tensor_id=i), threads=8)
        x = goq_inputs.activations_a16(1, inn, config_id=83, tensor_id=100 + i, outlier_frac=0.01)
        refs.append(oracle.gemm_a16(q, x, threads=8)[0])
        packed, xd = gu.pack_layer(goq, q), gu.to_dev(x.reshape(-1))
        y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        keep += [packed, xd]
        ys.append(y)
        probs.append((out, inn, packed, xd, None, y, goq.F32))
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    # eager call on the stream that will be captured: the stream gets its scratch region and the
    # library resolves what it resolves once per device, none of which may happen under capture
    with torch.cuda.stream(side):
        goq.gemv_batch(3, goq.A16, probs)
    side.synchronize()
    eager = [y.clone() for y in ys]
    for y, ref in zip(eager, refs):
        e1, _ = gu.a16_errors(y.cpu().numpy(), ref, None)
        assert e1 <= 1e-3, e1
    print("graph capture: %s" % kernel_name, flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        goq.gemv_batch(3, goq.A16, probs)
    for rep in range(3):
        for y in ys:
            y.fill_(float("nan"))                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(eager, ys)):
            assert torch.equal(a, b), (rep, k)
