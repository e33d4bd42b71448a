"""goq_pack on the GPU: the packed bytes against a packer written here from the layout's
description (csrc/goq_layout.h), and the goq_pack -> goq_unpack round trip; bit-exact, both bit
widths, ragged row counts."""
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


def _pack_by_the_book(q):
    """The packed buffer as csrc/goq_layout.h describes it, in plain numpy loops over (row block,
    macro-block, chunk, row, dword)."""
    bw = q["bw"]
    out, inn = q["codes"].shape
    gn, rbn, ch = inn // 128, (out + 63) // 64, (4 if bw == 3 else 5)
    zero = (1 << (bw - 1)) - 1
    buf = np.zeros(rbn * gn * ch * 64 * 4, np.uint32)
    for R in range(rbn):
        for g in range(gn):
            for r in range(64):
                row = 64 * R + r
                live = row < out
                codes = q["codes"][row, 128 * g:128 * g + 128].astype(np.uint32) if live else np.full(128, zero, np.uint32)
                pat = q["pattern"][row, 16 * g:16 * g + 16].astype(np.uint32) if live else np.zeros(16, np.uint32)
                sg = q["signs"][row, 16 * g:16 * g + 16].astype(np.uint32) if live else np.zeros(16, np.uint32)
                cw = (int(q["c1"][row, g]) | (int(q["c2"][row, g]) << 16)) if live else 0
                for h in range(4):
                    for d in range(4):
                        m = 4 * h + d
                        w = 0
                        for j in range(4):
                            lo, hi = int(codes[8 * m + j]), int(codes[8 * m + j + 4])
                            w |= ((lo | (hi << 3)) if bw == 3 else (lo | (hi << 4))) << (8 * j)
                        if bw == 3:
                            aux = [int(pat[m]), int(sg[m]) & 3, int(sg[m]) >> 2, (cw >> (30 - 2 * m)) & 3]
                            for j in range(4):
                                w |= aux[j] << (8 * j + 6)
                        buf[((((R * gn + g) * ch + h) * 64 + r) * 4) + d] = w
                if bw == 4:
                    for d in range(4):
                        w = ((cw >> (8 * d)) & 0xFF) << 24
                        for i in range(4):
                            m = 4 * d + i
                            w |= (int(pat[m]) | (int(sg[m]) << 2)) << (6 * i)
                        buf[((((R * gn + g) * ch + 4) * 64 + r) * 4) + d] = w
    return buf


@pytest.mark.parametrize("bw", [3, 4])
@pytest.mark.parametrize("shape", [(1, 128), (70, 256), (130, 384)])
def test_pack_matches_the_documented_layout(bw, shape):
    import paper_2605_26092_amd as goq
    out, inn = shape
    q = goq_inputs.canonical_random(bw, out, inn, config_id=23, tensor_id=out)
    packed = gu.pack_layer(goq, q).cpu().numpy().view(np.uint32)
    assert np.array_equal(packed, _pack_by_the_book(q))
