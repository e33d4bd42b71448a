"""goq_pack -> goq_unpack round trip on the GPU, bit-exact, both bit widths, ragged row counts."""
import numpy as np
import pytest

import goq_inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 128), (64, 128), (65, 256), (200, 384), (1100, 512)])
def test_pack_roundtrip(bw, shape):
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    out, inn = shape
    print("pack roundtrip bw=%d out=%d in=%d" % (bw, out, inn), flush=True)
    q = goq_inputs.canonical_random(bw, out, inn, config_id=21, tensor_id=out)
    packed = gu.pack_layer(goq, q)
    assert packed.numel() == goq.packed_bytes(bw, out, inn)
    back = {k: torch.zeros_like(gu.to_dev(q[k])) for k in ("codes", "pattern", "signs", "c1", "c2")}
    goq.unpack(bw, out, inn, packed, back["codes"], back["pattern"], back["signs"], back["c1"], back["c2"])
    torch.cuda.synchronize()
    for k in ("codes", "pattern", "signs"):
        assert np.array_equal(back[k].cpu().numpy(), q[k]), k
    for k in ("c1", "c2"):
        assert np.array_equal(back[k].cpu().numpy().view(np.uint16), q[k]), k


def test_padding_rows_are_zero_valued():
    """Rows added to reach a multiple of 64 decode to exact zeros (checked through a second
    unpack with the padded row count)."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    q = goq_inputs.canonical_random(3, 70, 128, config_id=22)
    packed = gu.pack_layer(goq, q)
    codes = torch.zeros((128, 128), dtype=torch.uint8, device="cuda")
    pat = torch.zeros((128, 16), dtype=torch.uint8, device="cuda")
    sg = torch.zeros((128, 16), dtype=torch.uint8, device="cuda")
    c1 = torch.zeros((128, 1), dtype=torch.int16, device="cuda")
    c2 = torch.zeros((128, 1), dtype=torch.int16, device="cuda")
    goq.unpack(3, 128, 128, packed, codes, pat, sg, c1, c2)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy()[:70], q["codes"])
    assert np.all(codes.cpu().numpy()[70:] == 3) and np.all(c1.cpu().numpy()[70:] == 0)
    assert np.all(c2.cpu().numpy()[70:] == 0) and np.all(pat.cpu().numpy()[70:] == 0)
