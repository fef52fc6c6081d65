"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

Only random draws and dtype conversion live here; nothing of the layer's
arithmetic.  Shapes and distributions stand in for RoBERTa-base / -large linear
layers: X, dY ~ N(0,1); W ~ N(0, 0.02^2) (bf16 configs) or N(0, 1/d_in) (the small
fp32 config); bf16 tensors are the round-to-nearest-even of the fp64 draw.
"""
import numpy as np
import torch

# name -> (n, d_in, d_out, k, dtype, seeds (X, W, dY), sketch seed)
CONFIGS = {
    "c1_fp32_small": dict(n=256, d_in=128, d_out=128, k=32, dtype="f32", seeds=(1001, 1002, 1003), seed=0x5EED0001),
    "c2_base_attn": dict(n=4096, d_in=768, d_out=768, k=410, dtype="bf16", seeds=(2001, 2002, 2003), seed=0x5EED0002),
    "c3_base_ffn_up": dict(n=4096, d_in=768, d_out=3072, k=410, dtype="bf16", seeds=(3001, 3002, 3003),
                           seed=0x5EED0003),
    "c3_base_ffn_down": dict(n=4096, d_in=3072, d_out=768, k=410, dtype="bf16", seeds=(3004, 3005, 3006),
                             seed=0x5EED0003),
    "c4_large_attn": dict(n=16384, d_in=1024, d_out=1024, k=1638, dtype="bf16", seeds=(4001, 4002, 4003),
                          seed=0x5EED0004),
    "c4_large_ffn_up": dict(n=16384, d_in=1024, d_out=4096, k=1638, dtype="bf16", seeds=(4004, 4005, 4006),
                            seed=0x5EED0004),
    "c4_large_ffn_down": dict(n=16384, d_in=4096, d_out=1024, k=1638, dtype="bf16", seeds=(4007, 4008, 4009),
                              seed=0x5EED0004),
}


def sketch_size(rho, n):
    """k = round(rho * n), at least 1 (410 for 0.1 * 4096, 1638 for 0.1 * 16384)."""
    return max(1, int(np.floor(rho * n + 0.5)))


def normal(shape, seed, std=1.0):
    """fp64 N(0, std^2) draw of the given shape from numpy's default_rng(seed)."""
    return np.random.default_rng(seed).standard_normal(shape) * std


def to_torch(a, dtype):
    """fp64 numpy -> CPU torch tensor of dtype "f32" / "bf16" (round to nearest even)."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.to(torch.float32 if dtype == "f32" else torch.bfloat16)


def to_f64(t):
    """Torch tensor (any device, fp32 / bf16) -> fp64 numpy, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def layer_inputs(n, d_in, d_out, dtype, seeds, w_std=None):
    """CPU tensors (X, W, dY) for one layer call."""
    if w_std is None:
        w_std = 0.02 if dtype == "bf16" else 1.0 / np.sqrt(d_in)
    X = to_torch(normal((n, d_in), seeds[0]), dtype)
    W = to_torch(normal((d_out, d_in), seeds[1], w_std), dtype)
    dY = to_torch(normal((n, d_out), seeds[2]), dtype)
    return X, W, dY


def config_inputs(name):
    c = CONFIGS[name]
    return layer_inputs(c["n"], c["d_in"], c["d_out"], c["dtype"], c["seeds"])


# ---------------------------------------------------------------------------------------------
# Config 5: a stack of 24 RoBERTa-large-shaped blocks of six isolated linear layers each
# (4 attention projections 1024 -> 1024, FFN 1024 -> 4096 and 4096 -> 1024), N = 16384 tokens,
# k = 1638.  Layer l (0 .. 143) uses the sketch state (seed 5000 + l, offset l).  Inputs come
# from a pool of three sets per shape (drawn with the seeds below): blocks 0-7 use set 0, blocks
# 8-15 set 1, blocks 16-23 set 2, so the first, the middle (block 12) and the last block see
# three different sets.  Drawing 144 independent sets (15 GB) on the host would take minutes
# and change nothing that is measured.
STACK = dict(blocks=24, n=16384, d=1024, d_ff=4096, k=1638, dtype="bf16", seed_base=5000, pool_seed_base=5100)


def stack_layers():
    """[(layer index, block, shape name, d_in, d_out, pool set, sketch seed, offset)] in forward order."""
    out = []
    for blk in range(STACK["blocks"]):
        for j in range(6):
            shape = "attn" if j < 4 else ("ffn_up" if j == 4 else "ffn_down")
            d_in = STACK["d_ff"] if shape == "ffn_down" else STACK["d"]
            d_out = STACK["d_ff"] if shape == "ffn_up" else STACK["d"]
            l = 6 * blk + j
            out.append(dict(layer=l, block=blk, shape=shape, d_in=d_in, d_out=d_out, pool=min(blk // 8, 2),
                            seed=STACK["seed_base"] + l, offset=l))
    return out


def stack_pool_inputs(shape, pool):
    """CPU tensors (X, W, dY) of pool set `pool` (0..2) for shape "attn" / "ffn_up" / "ffn_down"."""
    idx = ("attn", "ffn_up", "ffn_down").index(shape)
    d_in = STACK["d_ff"] if shape == "ffn_down" else STACK["d"]
    d_out = STACK["d_ff"] if shape == "ffn_up" else STACK["d"]
    s = STACK["pool_seed_base"] + 10 * idx + 3 * pool
    return layer_inputs(STACK["n"], d_in, d_out, STACK["dtype"], (s, s + 1, s + 2))


def pattern_rows(row0, rows, cols, mult, mod):
    """Deterministic bf16-exact test matrix block (no random draw, so a multi-GiB operand can be
    made in pieces on either side): entry (i, j) = ((mult * i + 7 * j) % mod - mod // 2) / 8."""
    i = np.arange(row0, row0 + rows, dtype=np.int64)[:, None]
    j = np.arange(cols, dtype=np.int64)[None, :]
    return ((mult * i + 7 * j) % mod - mod // 2).astype(np.float64) / 8.0
