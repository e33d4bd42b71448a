"""goq_gemv_batch, the batch-1 entry point for callers that cannot allocate (its scratch for split
row groups is a static device array inside the library), against goq_gemv_batch_ws, the same
kernels with a caller-owned workspace: equal bits, on two calls in a row, the second with a smaller
input (the static array keeps the first call's contents: what must start at zero has to be back at
zero).  Called through the C ABI (ctypes) directly.  Collected last on purpose."""
import ctypes

import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _descs(binding, problems):
    arr = (binding._Desc * len(problems))()
    for d, (out, inn, packed, x, y) in zip(arr, problems):
        d.out, d.in_, d.packed, d.x, d.sx, d.y, d.ytype = out, inn, packed.data_ptr(), x.data_ptr(), None, y.data_ptr(), binding.F32
    return arr


def test_static_scratch_entry_point_equals_workspace_entry_point(oracle):
    import paper_2605_26092_amd as goq
    from paper_2605_26092_amd import binding
    torch = gu.torch_cuda()
    L = goq.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.goq_gemv_select(binding.GEMV_STREAM) == 0        # the kernel that uses the scratch
    try:
        nbytes = ctypes.c_size_t(0)
        assert L.goq_gemv_workspace_bytes(ctypes.byref(nbytes)) == 0
        ws = torch.empty(nbytes.value + 256, dtype=torch.uint8, device="cuda")
        ws = ws[(-ws.data_ptr()) % 256:][:nbytes.value]
        assert L.goq_gemv_workspace_init(stream, ctypes.c_void_p(ws.data_ptr())) == 0

        # first call: three layers whose row groups are cut by many piece boundaries; second call:
        # a smaller input (fewer, smaller layers: other boundaries, fewer counters in use)
        calls = [[(1500, 2048), (700, 4096), (2100, 1024)], [(600, 1024), (130, 512)]]
        keep = []
        for ci, shapes in enumerate(calls):
            probs_a, probs_b, refs = [], [], []
            for i, (out, inn) in enumerate(shapes):
                q = oracle.quantize_geo(3, goq_inputs.weights(out, inn, config_id=70 + ci, tensor_id=i), threads=8)
                x = goq_inputs.activations_a16(1, inn, config_id=70 + ci, tensor_id=100 + i, outlier_frac=0.01)
                refs.append(oracle.gemm_a16(q, x, threads=8)[0])
                packed = gu.pack_layer(goq, q)
                xd = gu.to_dev(x.reshape(-1))
                ya = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
                yb = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
                keep += [packed, xd]
                probs_a.append((out, inn, packed, xd, ya))
                probs_b.append((out, inn, packed, xd, yb))
            da, db = _descs(binding, probs_a), _descs(binding, probs_b)
            print("no-alloc call %d: %s" % (ci, shapes), flush=True)
            rc = L.goq_gemv_batch(stream, 3, binding.A16, len(da), da)
            assert rc == 0, goq.last_error()
            rc = L.goq_gemv_batch_ws(stream, 3, binding.A16, len(db), db, ctypes.c_void_p(ws.data_ptr()))
            assert rc == 0, goq.last_error()
            torch.cuda.synchronize()
            for (_, _, _, _, ya), (_, _, _, _, yb), ref in zip(probs_a, probs_b, refs):
                assert torch.equal(ya, yb)
                e1, _ = gu.a16_errors(ya.cpu().numpy(), ref, None)
                assert e1 <= 1e-3, e1
    finally:
        L.goq_gemv_select(binding.GEMV_AUTO)
