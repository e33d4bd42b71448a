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


# ---- the whole block of every GEMM config through the batch entry point bench.py times ------------

def _quantize_block(goq, oracle, bw, block, cid):
    """Seeded weights of every matrix of the block (drawn in parallel threads: the generators are
    independent), quantised by the oracle one after the other, packed on the device."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=len(block)) as pool:
        Ws = list(pool.map(lambda a: goq_inputs.weights(a[1][1], a[1][2], config_id=cid, tensor_id=a[0]), enumerate(block)))
    packed, canon = [], []
    for idx, (name, out, inn) in enumerate(block):
        print("  quantise %s %dx%d (bw %d)" % (name, out, inn, bw), flush=True)
        q = oracle.quantize_geo(bw, Ws[idx], threads=16)
        Ws[idx] = None
        packed.append(gu.pack_layer(goq, q))
        canon.append(q)
    return packed, canon


@pytest.mark.parametrize("bw", [3, 4])
def test_config3_block_gemm_batch_full_size(oracle, bw):
    """BASELINE config 3: all seven LLaMA-2-7B block matrices, 2048 tokens, W3/A16 and W4/A16, as
    the ONE goq_gemm_batch launch bench.py times (fp16 outputs); the oracle checks a seeded sample
    of 8 token rows over all outputs of every matrix."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    tokens = 2048
    print("config3 block bw=%d" % bw, flush=True)
    packed, canon = _quantize_block(goq, oracle, bw, goq_inputs.LLAMA2_7B_BLOCK, 3)
    Xs, Ys, probs = [], [], []
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_7B_BLOCK):
        X = goq_inputs.activations_a16(tokens, inn, config_id=3, tensor_id=100 + idx, outlier_frac=0.01)
        Xs.append(X)
        Y = torch.full((tokens, out), float("nan"), dtype=torch.float16, device="cuda")
        Ys.append(Y)
        probs.append((tokens, out, inn, packed[idx], gu.to_dev(X), None, Y, goq.F16))
    goq.gemm_batch(bw, goq.A16, probs)
    torch.cuda.synchronize()
    rows = np.sort(goq_inputs.rng(3, 998).choice(tokens, size=8, replace=False))
    ridx = torch.from_numpy(rows).cuda()
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_7B_BLOCK):
        assert not torch.isnan(Ys[idx].float()).any(), name
        ref = oracle.gemm_a16(canon[idx], Xs[idx][rows], threads=16)
        y = Ys[idx][ridx].float().cpu().numpy().astype(np.float64)
        e1, _ = gu.a16_errors(y, ref, None)
        print("  %s: max rel err %.3g" % (name, e1), flush=True)
        assert e1 <= TOL, (name, e1)


def test_config4_block_gemm_batch_full_size(oracle):
    """BASELINE config 4: all four ViT-B block matrices, 197 x 64 tokens, W3/A8, as ONE goq_gemm_batch
    launch.  With the partials output: int32 slab partials bit-exact on a seeded sample of 24 token
    rows, all outputs, all slabs, every matrix.  Then the launch exactly as bench.py times it (fp16
    outputs, no partials), held to the fp16 rounding of the oracle's result."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    tokens = 197 * 64
    print("config4 block", flush=True)
    packed, canon = _quantize_block(goq, oracle, 3, goq_inputs.VIT_B_BLOCK, 4)
    Xq, sxs, Ys, Ps, probs, probs_bench, Yb = [], [], [], [], [], [], []
    for idx, (name, out, inn) in enumerate(goq_inputs.VIT_B_BLOCK):
        xq, sx = goq_inputs.activations_a8(tokens, inn, config_id=4, tensor_id=200 + idx)
        Xq.append(xq)
        sxs.append(sx)
        Xd, sxd = gu.to_dev(xq), gu.to_dev(sx)
        Y = torch.full((tokens, out), float("nan"), dtype=torch.float32, device="cuda")
        P = torch.full((tokens, out, inn // 128, 2), -7, dtype=torch.int32, device="cuda")
        Y16 = torch.full((tokens, out), float("nan"), dtype=torch.float16, device="cuda")
        Ys.append(Y)
        Ps.append(P)
        Yb.append(Y16)
        probs.append((tokens, out, inn, packed[idx], Xd, sxd, Y, goq.F32, P))
        probs_bench.append((tokens, out, inn, packed[idx], Xd, sxd, Y16, goq.F16))
    goq.gemm_batch(3, goq.A8, probs)
    goq.gemm_batch(3, goq.A8, probs_bench)
    torch.cuda.synchronize()
    rows = np.sort(goq_inputs.rng(4, 998).choice(tokens, size=24, replace=False))
    ridx = torch.from_numpy(rows).cuda()
    for idx, (name, out, inn) in enumerate(goq_inputs.VIT_B_BLOCK):
        ref, rp = oracle.gemm_a8(canon[idx], Xq[idx][rows], sxs[idx][rows], threads=16, want_partials=True)
        assert np.array_equal(Ps[idx][ridx].cpu().numpy(), rp), name
        y = Ys[idx][ridx].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(y - ref)) <= 1e-5 * np.max(np.abs(ref)), name
        assert not torch.isnan(Yb[idx].float()).any(), name
        y16 = Yb[idx][ridx].float().cpu().numpy().astype(np.float64)
        e1, _ = gu.a16_errors(y16, ref, None)
        assert e1 <= TOL, (name, e1)
        # the fp16 launch rounds the same fp32 values
        assert torch.equal(Yb[idx][ridx], Ys[idx][ridx].half()), name


def test_config5_layer_gemv_batch_and_gemm_batch_full_size(oracle):
    """BASELINE config 5: all seven LLaMA-2-70B layer matrices (856 M weights) on one GPU, W3/A16.
    The seven GEMVs as ONE goq_gemv_batch launch (every output against the oracle) and the
    512-token GEMMs as ONE goq_gemm_batch launch (a seeded sample of 4 token rows over all outputs
    of every matrix): the two launches bench.py times."""
    import paper_2605_26092_amd as goq
    torch = gu.torch_cuda()
    tokens = 512
    print("config5 layer", flush=True)
    packed, canon = _quantize_block(goq, oracle, 3, goq_inputs.LLAMA2_70B_LAYER, 5)
    probs, ys, xs = [], [], []
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_70B_LAYER):
        x = goq_inputs.activations_a16(1, inn, config_id=5, tensor_id=100 + idx, outlier_frac=0.01)
        xs.append(x)
        y = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
        ys.append(y)
        probs.append((out, inn, packed[idx], gu.to_dev(x.reshape(-1)), None, y, goq.F32))
    for rep in range(2):
        goq.gemv_batch(3, goq.A16, probs)
    torch.cuda.synchronize()
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_70B_LAYER):
        ref = oracle.gemm_a16(canon[idx], xs[idx], threads=16)[0]
        e1, _ = gu.a16_errors(ys[idx].cpu().numpy(), ref, None)
        print("  gemv %s: max rel err %.3g" % (name, e1), flush=True)
        assert e1 <= TOL, (name, e1)
    Xs, Ys, gprobs = [], [], []
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_70B_LAYER):
        X = goq_inputs.activations_a16(tokens, inn, config_id=5, tensor_id=300 + idx, outlier_frac=0.01)
        Xs.append(X)
        Y = torch.full((tokens, out), float("nan"), dtype=torch.float16, device="cuda")
        Ys.append(Y)
        gprobs.append((tokens, out, inn, packed[idx], gu.to_dev(X), None, Y, goq.F16))
    goq.gemm_batch(3, goq.A16, gprobs)
    torch.cuda.synchronize()
    rows = np.sort(goq_inputs.rng(5, 998).choice(tokens, size=4, replace=False))
    ridx = torch.from_numpy(rows).cuda()
    for idx, (name, out, inn) in enumerate(goq_inputs.LLAMA2_70B_LAYER):
        assert not torch.isnan(Ys[idx].float()).any(), name
        ref = oracle.gemm_a16(canon[idx], Xs[idx][rows], threads=16)
        y = Ys[idx][ridx].float().cpu().numpy().astype(np.float64)
        e1, _ = gu.a16_errors(y, ref, None)
        print("  gemm %s: max rel err %.3g" % (name, e1), flush=True)
        assert e1 <= TOL, (name, e1)
