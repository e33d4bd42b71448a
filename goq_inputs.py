"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path.

Holds none of the method's arithmetic: only random tensors with the shapes and value
statistics of the workloads (LLaMA-2-7B / 70B and ViT-B shaped linear layers), which
stand in for the checkpoints and activations the paper evaluates on.

  weights      N(0, 0.02^2), 0.5 % of entries redrawn from 0.02 * Student-t(nu=4), cast to fp16
  A16 inputs   fp16 N(0,1); optionally round(frac * in) channels scaled by 20 for every token
  A8 inputs    N(0,1) per element, per-token symmetric int8: s_x = max|x| / 127,
               x~ = clip(rint(x / s_x), -127, 127)   (round-half-even)
  canonical    codes / pattern / signs / coefficients drawn directly from a stated
               distribution, for full-size throughput runs where the values do not matter
"""
import numpy as np

N = 128
G = 8

# (name, out, in)
LLAMA2_7B_BLOCK = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                   ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA2_70B_LAYER = [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
                    ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]
VIT_B_BLOCK = [("qkv", 2304, 768), ("proj", 768, 768), ("fc1", 3072, 768), ("fc2", 768, 3072)]


def rng(config_id, tensor_id):
    return np.random.default_rng(np.random.SeedSequence([int(config_id), int(tensor_id)]))


def weights(out, inn, config_id=0, tensor_id=0):
    """fp16 weights [out, in]."""
    r = rng(config_id, tensor_id)
    w = r.normal(0.0, 0.02, size=(out, inn))
    mask = r.random(size=(out, inn)) < 0.005
    t = 0.02 * r.standard_t(4, size=int(mask.sum()))
    w[mask] = t
    return w.astype(np.float16)


def activations_a16(tokens, inn, config_id=0, tensor_id=100, outlier_frac=0.0):
    """fp16 activations [tokens, in]; outlier channels are scaled by 20 for every token."""
    r = rng(config_id, tensor_id)
    x = r.normal(0.0, 1.0, size=(tokens, inn))
    n_out = int(round(outlier_frac * inn))
    if n_out > 0:
        ch = r.choice(inn, size=n_out, replace=False)
        x[:, ch] *= 20.0
    return x.astype(np.float16)


def activations_a8(tokens, inn, config_id=0, tensor_id=200):
    """(int8 [tokens, in], float32 scale [tokens])."""
    r = rng(config_id, tensor_id)
    x = r.normal(0.0, 1.0, size=(tokens, inn))
    sx = (np.abs(x).max(axis=1) / 127.0).astype(np.float32)
    sx[sx == 0] = 1.0
    xq = np.clip(np.rint(x / sx[:, None].astype(np.float64)), -127, 127).astype(np.int8)
    return xq, sx


def activations_int(tokens, inn, bits, config_id=0, tensor_id=200):
    """b_a-bit per-token symmetric integer activations in int8 containers (the paper's A3..A6
    operating points): (int8 [tokens, in] with |x| <= 2^(bits-1) - 1, float32 scale [tokens])."""
    r = rng(config_id, tensor_id)
    x = r.normal(0.0, 1.0, size=(tokens, inn))
    top = float((1 << (bits - 1)) - 1)
    sx = (np.abs(x).max(axis=1) / top).astype(np.float32)
    sx[sx == 0] = 1.0
    xq = np.clip(np.rint(x / sx[:, None].astype(np.float64)), -top, top).astype(np.int8)
    return xq, sx


def pack_int4(xq):
    """int8 values in [-8, 7], [tokens, in] -> packed int4 bytes [tokens, in / 2]: element 2 i in
    the low nibble of byte i, two's complement (storage format only, no arithmetic)."""
    u = (xq.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


def pack_int6(xq):
    """int8 values in [-32, 31], [tokens, in] -> packed int6 bytes [tokens, 3 in / 4]: element k in
    bits 6 k .. 6 k + 5 of the row read as a little-endian bit string, two's complement (storage
    format only, no arithmetic)."""
    u = (xq.astype(np.int32) & 0x3F).astype(np.uint32)
    w = u[:, 0::4] | (u[:, 1::4] << 6) | (u[:, 2::4] << 12) | (u[:, 3::4] << 18)      # 24 bits per four elements
    out = np.empty((xq.shape[0], xq.shape[1] // 4, 3), dtype=np.uint8)
    out[:, :, 0] = w & 0xFF
    out[:, :, 1] = (w >> 8) & 0xFF
    out[:, :, 2] = (w >> 16) & 0xFF
    return out.reshape(xq.shape[0], -1)


def pack_int3(xq):
    """int8 values in [-4, 3], [tokens, in] -> packed int3 bytes [tokens, 3 in / 8]: element k in
    bits 3 k .. 3 k + 2 of the row read as a little-endian bit string, two's complement (storage
    format only, no arithmetic)."""
    u = (xq.astype(np.int32) & 0x7).astype(np.uint32)
    w = np.zeros((xq.shape[0], xq.shape[1] // 8), dtype=np.uint32)
    for i in range(8):
        w |= u[:, i::8] << (3 * i)                                                # 24 bits per eight elements
    out = np.empty((xq.shape[0], xq.shape[1] // 8, 3), dtype=np.uint8)
    out[:, :, 0] = w & 0xFF
    out[:, :, 1] = (w >> 8) & 0xFF
    out[:, :, 2] = (w >> 16) & 0xFF
    return out.reshape(xq.shape[0], -1)


# W3 code histogram measured by quantising `weights()` with the GEO quantizer; codes follow the
# canonical numbering (0:+1, 1:+.5, 2:+.25, 3:0, 4:-1, 5:-.5, 6:-.25, 7:-.125).
_W3_HIST = np.array([0.0205, 0.1249, 0.2153, 0.2104, 0.0202, 0.1251, 0.1511, 0.1324])
# W4: codes 0..6 = +2^0..+2^-6, 7 = 0, 8..15 = -2^0..-2^-7.
_W4_HIST = np.array([0.0205, 0.1249, 0.1513, 0.0977, 0.0523, 0.0266, 0.0178, 0.0134,
                     0.0202, 0.1251, 0.1511, 0.0976, 0.0526, 0.0266, 0.0133, 0.0089])


def canonical_random(bw, out, inn, config_id=0, tensor_id=300):
    """Canonical arrays drawn directly (no quantizer): dict like the quantizer's output."""
    r = rng(config_id, tensor_id)
    hist = _W3_HIST if bw == 3 else _W4_HIST
    codes = r.choice(1 << bw, size=(out, inn), p=hist / hist.sum()).astype(np.uint8)
    pattern = r.integers(0, 4, size=(out, inn // G), dtype=np.uint8)
    signs = r.integers(0, 16, size=(out, inn // G), dtype=np.uint8)
    c1 = np.abs(r.normal(0.056, 0.01, size=(out, inn // N))).astype(np.float16)
    c2 = np.abs(r.normal(0.008, 0.003, size=(out, inn // N))).astype(np.float16)
    return {"bw": bw, "codes": codes, "pattern": pattern, "signs": signs,
            "c1": c1.view(np.uint16), "c2": c2.view(np.uint16)}
