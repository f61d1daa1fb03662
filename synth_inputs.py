"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

Holds no arithmetic of the method: only random draws and the shapes of the
workloads.  The draws stand in for TriLM layers whose trained weights are not
available here: ternary weights iid with P(-1) = P(+1) = 0.3, P(0) = 0.4,
activations fp16 ~ N(0, 1), one fp16 scale per matrix.
"""
import numpy as np

P_NEG = 0.3
P_POS = 0.3

# name -> (K, N): Llama-style layer shapes the workloads are quoted on.
SHAPES = {
    "sq2048": (2048, 2048),
    "attn_o": (4096, 4096),          # hidden 4096 -> 4096
    "mlp_up_8b": (4096, 14336),      # hidden 4096 -> MLP 14336
    "qkv": (4096, 12288),
    "gate_up": (4096, 22016),        # SwiGLU gate+up, MLP 11008
    "down": (11008, 4096),
}

SEEDS = {"c1": 23025001, "c2": 23025002, "c3": 23025003, "c4": 23025004, "c5": 23025005}

DECODE_SWEEP_M = (1, 2, 4, 8, 16)
DECODE_SWEEP_SHAPES = ("attn_o", "mlp_up_8b")
BLOCK_SHAPES = ("qkv", "attn_o", "gate_up", "down")
BLOCK_M = (1, 16, 64)
PREFILL_M = (256, 1024, 2048)


def ternary_weights(rng, N, K, p_neg=P_NEG, p_pos=P_POS):
    """int8 [N][K] with values -1 / 0 / +1 drawn iid."""
    u = rng.random((N, K), dtype=np.float32)
    W = np.zeros((N, K), dtype=np.int8)
    W[u < p_neg] = -1
    W[u >= 1.0 - p_pos] = 1
    return W


def activations(rng, M, K):
    """fp16 [M][K] ~ N(0, 1)."""
    return rng.standard_normal((M, K), dtype=np.float32).astype(np.float16)


def gamma_fixed(value=0.02):
    return np.float16(value)


def gamma_uniform(rng, lo=0.01, hi=0.05):
    """One scale per matrix: drawn in fp64, rounded to fp16 before anyone uses it."""
    return np.float16(rng.uniform(lo, hi))


def group_scales(rng, groups, N, lo=0.01, hi=0.05):
    """fp16 [groups][N]: one scale per group of weights along K and output row, drawn in fp64
    and rounded to fp16 before anyone uses it."""
    return rng.uniform(lo, hi, size=(groups, N)).astype(np.float16)


def gamma_bits(g):
    return int(np.array(g, dtype=np.float16).view(np.uint16))


def layer(seed, M, N, K, fixed_gamma=None):
    """(x fp16 [M][K], W int8 [N][K], gamma fp16) for one linear layer."""
    rng = np.random.default_rng(seed)
    W = ternary_weights(rng, N, K)
    x = activations(rng, M, K)
    g = gamma_fixed(fixed_gamma) if fixed_gamma is not None else gamma_uniform(rng)
    return x, W, g
