"""Seeded synthetic inputs with the shapes and statistics of the DiT-XL/2 linear stack.

This module holds NONE of the method's arithmetic: no quantizer, no GEMM, no
dequantization.  It only draws tensors.  Both the CPU oracle's tests and the HIP
path's tests/benchmark take their inputs from here, so the two sides always see
identical bits.

What stands in for what: the paper measures a class-conditional DiT-XL/2 on
image datasets (Section 6).  Neither trained weights nor those datasets are
used here; only shapes (hidden 1152, MLP 4608, 28 blocks, 256 tokens per
256-pixel image, 1024 per 512-pixel image) and the qualitative statistics the
paper describes are kept: a few outlier channels ("channel imbalance",
Section 1) and an activation standard deviation that drifts over the denoising
trajectory (Step 3, activation-statistics figures).
"""
import hashlib

import numpy as np

SEED = 251111446

HIDDEN = 1152
MLP = 4608
N_BLOCKS = 28

# name -> (K_in, N_out) of the four quantized linears of one DiT block (Step 3:
# DAQ sits at the inputs of Q/K/V, the attention output projection and both MLP layers)
BLOCK_LAYERS = (("qkv", HIDDEN, 3 * HIDDEN), ("proj", HIDDEN, HIDDEN), ("fc1", HIDDEN, MLP), ("fc2", MLP, HIDDEN))


def rng(*key):
    """Counter-based generator keyed by (SEED, *key); independent streams per key."""
    h = hashlib.sha256(repr((SEED,) + tuple(key)).encode()).digest()
    k = np.frombuffer(h[:16], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=k))


def outlier_channels(K, n_outlier, *key):
    return np.sort(rng("outlier", K, *key).choice(K, size=min(n_outlier, K), replace=False))


def activations(M, K, *key, sigma=1.0, n_outlier=8, outlier_gain=20.0):
    """fp16 [M,K]: N(0, sigma^2) with n_outlier seeded channels multiplied by outlier_gain."""
    g = rng("act", M, K, *key)
    z = g.standard_normal((M, K), dtype=np.float32)
    c = np.ones((K,), np.float32)
    if n_outlier:
        c[outlier_channels(K, n_outlier, *key)] = outlier_gain
    return (z * c * np.float32(sigma)).astype(np.float16)


def gelu_tanh_f16(y):
    """fp16 -> fp16 tanh-GELU; used only to shape the input of fc2 like an MLP hidden state."""
    v = y.astype(np.float32)
    out = 0.5 * v * (1.0 + np.tanh(0.7978845608028654 * (v + 0.044715 * v * v * v)))
    return out.astype(np.float16)


def w8_codes(N, K, *key):
    """int8 [N,K] iid uniform integers in [-127, 127]."""
    return rng("w8", N, K, *key).integers(-127, 128, size=(N, K), dtype=np.int8)


def w8_scales(N, *key):
    """fp32 [N] ~ U(1e-3, 1e-2): one scale per output channel."""
    return rng("w8s", N, *key).uniform(1e-3, 1e-2, size=(N,)).astype(np.float32)


def w4_codes(N, K, *key):
    """int8 [N,K] iid uniform integers in [-8, 7] (to be packed two per byte)."""
    return rng("w4", N, K, *key).integers(-8, 8, size=(N, K), dtype=np.int8)


def w4_scales(N, K, *key):
    """fp16 [N, K/128] ~ U(1e-2, 1e-1): one scale per output channel per group of 128 inputs."""
    return rng("w4s", N, K, *key).uniform(1e-2, 1e-1, size=(N, K // 128)).astype(np.float16)


def w4_scales_group(N, K, group, *key):
    """fp16 [N, K/group] ~ U(1e-2, 1e-1) for weight groups of `group` inputs (the plan's other group sizes)."""
    return rng("w4sg", N, K, group, *key).uniform(1e-2, 1e-1, size=(N, K // group)).astype(np.float16)


def bias(N, *key):
    """fp16 [N] ~ N(0, 0.02^2)."""
    return (rng("bias", N, *key).standard_normal((N,), dtype=np.float32) * np.float32(0.02)).astype(np.float16)


def sigma_schedule(steps, hi=5.0, lo=0.2):
    """Per-timestep activation std, geometric from hi (early, volatile) down to lo (late, stable)."""
    if steps == 1:
        return np.array([hi])
    i = np.arange(steps, dtype=np.float64)
    return hi * (lo / hi) ** (i / (steps - 1))


def bit_plan(n_blocks=N_BLOCKS, p_w4=77.0 / 91.0, protect=3, *key):
    """Seeded per-layer weight-bit plan over the 4*n_blocks block linears.

    The paper's final plan keeps 77 layers at W4 and 14 at W8 among the quantized
    layers (Step 2) and treats the first and last blocks as fragile; here each
    layer is W4 with probability p_w4, except that the first and last `protect`
    blocks stay W8.  Returns a list of dicts(name, block, K, N, bits, group).
    """
    g = rng("plan", n_blocks, *key)
    plan = []
    for b in range(n_blocks):
        for name, K, N in BLOCK_LAYERS:
            fragile = b < protect or b >= n_blocks - protect
            bits = 8 if fragile or g.random() >= p_w4 else 4
            plan.append(dict(name=name, block=b, K=K, N=N, bits=bits, group=128 if bits == 4 else 0))
    return plan


def final_plan(n_blocks=N_BLOCKS, *key):
    """The kind of plan the paper ends Step 2 with, over the 4*n_blocks block linears: of its 113 layers 77 are W4,
    14 W8 and 22 FP16, with group sizes 288 (86 layers), 64 (9), 128 (5), 192 (6) and 32 (7).  The 113th layer (the final
    projection) is not a block linear; it is taken to be one of the FP16, group-288 entries.  Which layer gets which
    entry is a seeded shuffle (the paper does not list them).  Returns dicts(name, block, K, N, bits, group)."""
    g = rng("final-plan", n_blocks, *key)
    n = 4 * n_blocks
    bits = [4] * 77 + [8] * 14 + [16] * 21
    groups = [288] * 85 + [64] * 9 + [128] * 5 + [192] * 6 + [32] * 7
    if n != len(bits):      # other depths: same proportions
        bits = [bits[i * len(bits) // n] for i in range(n)]
        groups = [groups[i * len(groups) // n] for i in range(n)]
    bits = [bits[i] for i in g.permutation(n)]
    groups = [groups[i] for i in g.permutation(n)]
    plan, i = [], 0
    for b in range(n_blocks):
        for name, K, N in BLOCK_LAYERS:
            plan.append(dict(name=name, block=b, K=K, N=N, bits=bits[i], group=groups[i] if bits[i] == 4 else 0))
            i += 1
    return plan


def f16_weights(N, K, *key):
    """fp16 [N,K] ~ N(0, 0.02^2): the weights of a layer the plan leaves unquantized."""
    return (rng("w16", N, K, *key).standard_normal((N, K), dtype=np.float32) * np.float32(0.02)).astype(np.float16)


# Workloads (rows M, DAQ rows-per-scale R, layers, steps); the keys match the
# benchmark's --workload flag.
WORKLOADS = {
    # single W8A8 linear, one 256-token image, per-tensor scale
    "c1_single_w8a8": dict(M=256, R=256, steps=1, layers=[("proj", HIDDEN, HIDDEN, 8)]),
    # one block, 8 images x 256 tokens, per-token
    "c2_block_w8a8_m2048": dict(M=2048, R=1, steps=1, layers=[(n, k, o, 8) for n, k, o in BLOCK_LAYERS]),
    # mixed: MLP layers int4 group-128, attention layers int8; 32 images
    "c3_block_mixed_m8192": dict(M=8192, R=1, steps=1,
                                 layers=[("qkv", HIDDEN, 3 * HIDDEN, 8), ("proj", HIDDEN, HIDDEN, 8),
                                         ("fc1", HIDDEN, MLP, 4), ("fc2", MLP, HIDDEN, 4)]),
    # 512-pixel shapes: 16 images x 1024 tokens, 50 drifting timesteps
    "c4_block_w8a8_m16384": dict(M=16384, R=1, steps=50, layers=[(n, k, o, 8) for n, k, o in BLOCK_LAYERS]),
    # the full 28-block stack under a seeded bit plan, 64 images x 256 tokens, 25 timesteps
    "c5_stack_plan_m16384": dict(M=16384, R=1, steps=25, layers="bit_plan"),
    # the same stack under a plan of the paper's final kind: W4 with mixed group sizes, W8 and FP16 layers
    "c6_stack_final_plan_m16384": dict(M=16384, R=1, steps=25, layers="final_plan"),
}


def layer_weights(name, K, N, bits, *key):
    """Weights, scales and bias of one layer: dict(bits, w (int8 codes [N,K]), s_w, bias)."""
    if bits == 8:
        return dict(bits=8, w=w8_codes(N, K, name, *key), s_w=w8_scales(N, name, *key), bias=bias(N, name, *key))
    if bits == 4:
        return dict(bits=4, w=w4_codes(N, K, name, *key), s_w=w4_scales(N, K, name, *key), bias=bias(N, name, *key))
    if bits == 16:
        return dict(bits=16, w=f16_weights(N, K, name, *key), s_w=None, bias=bias(N, name, *key))
    raise ValueError("bits must be 4, 8 or 16")
