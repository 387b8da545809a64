"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors on the host (CPU generator, so the bytes
are the same on every machine).  It contains none of the method's arithmetic
and is the one piece the tests hand to both the HIP path and the CPU oracle.

The paper trains Gemma-2 2B / 9B and Mistral 7B feed-forward weights on C4
tokens (section 4, appendix B).  Neither the weights nor the data are
available, so each configuration draws a seeded layer of the same shape with a
stated value distribution.

Every tensor has its own generator seeded from (config seed, tensor name), so
any single tensor can be regenerated without drawing the others.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field

import torch

# (N, K) = (output channels, input features) of each linear of the MLP.
_MLP = {
    2: dict(d_model=2304, ffn=9216, tokens=4096),   # Gemma-2-2B-shaped
    3: dict(d_model=3584, ffn=14336, tokens=8192),  # Gemma-2-9B-shaped
    5: dict(d_model=4608, ffn=36864, tokens=4096),  # Gemma-2-27B-shaped
}
# Decode shapes (K -> N) of the 7B-shaped model.
DECODE_SHAPES = [(4096, 4096), (14336, 4096), (4096, 14336)]  # (N, K)
DECODE_BATCHES = [1, 4, 16]

LAMBDAS = {1: (1.0, 1.0, 1.0), 2: (1.0, 1.0, 1.0), 3: (0.1, 0.1, 1.0), 5: (1.0, 1.0, 1.0)}


def config_seed(config: int) -> int:
    return config - 1


def _gen(config: int, name: str) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(config_seed(config) * 1_000_003 + zlib.crc32(name.encode()))
    return g


def mlp_shapes(config: int):
    """{'gate': (N, K), 'up': (N, K), 'down': (N, K)} and the token count."""
    c = _MLP[config]
    d, f = c["d_model"], c["ffn"]
    return {"gate": (f, d), "up": (f, d), "down": (d, f)}, c["tokens"]


def weight(config: int, name: str, shape=None) -> torch.Tensor:
    """fp32 master weight [N, K] of linear `name` for `config`."""
    g = _gen(config, "W:" + name)
    if config == 1:
        N, K = shape or (256, 256)
        return torch.randn(N, K, generator=g) * 0.02
    if config == 2:
        N, K = shape or mlp_shapes(2)[0][name]
        return torch.randn(N, K, generator=g) * 0.02
    if config == 3:
        N, K = shape or mlp_shapes(3)[0][name]
        W = torch.randn(N, K, generator=g) * 0.015
        mask = torch.rand(N, K, generator=g) < 1e-3  # 0.1 % of entries become outliers
        W[mask] *= 8.0
        return W
    if config == 4:
        N, K = shape
        return torch.randn(N, K, generator=g) * 0.02
    if config == 5:
        # Student-t with 3 degrees of freedom: z0 / sqrt((z1^2 + z2^2 + z3^2) / 3).
        N, K = shape or mlp_shapes(5)[0][name]
        num = torch.randn(N, K, generator=g)
        den = torch.zeros(N, K)
        for _ in range(3):
            den += torch.randn(N, K, generator=g).square_()
        den.div_(3.0).sqrt_()
        return num.div_(den).mul_(0.01)
    raise ValueError(config)


def activations(config: int, name: str, M: int, K: int) -> torch.Tensor:
    """bf16 activations [M, K] ~ N(0, 1)."""
    return torch.randn(M, K, generator=_gen(config, "X:" + name)).to(torch.bfloat16)


def out_grads(config: int, name: str, M: int, N: int, nr: int = 3):
    """nr bf16 output gradients [M, N] ~ N(0, 1e-3^2), one per bit-width."""
    return [(torch.randn(M, N, generator=_gen(config, f"dY{i}:" + name)) * 1e-3).to(torch.bfloat16)
            for i in range(nr)]


def uniform_codes(seed: int, N: int, K: int) -> torch.Tensor:
    """int8 codes uniform on 0..255: the extra-precision density sweep's dense end."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randint(0, 256, (N, K), generator=g, dtype=torch.int32).to(torch.uint8)


def planted_codes(seed: int, N: int, K: int, first_hot: int, frac: float) -> torch.Tensor:
    """int8 codes in which a Bernoulli(frac) subset is uniform on first_hot..255 and the rest uniform on
    0..first_hot-1.

    The caller chooses `first_hot` (the tests pass the first code of the overflow bucket of the slice they
    exercise: the paper's trained extra-precision models put about 2-5 % of the weights there, Table 7,
    while min-max quantized random weights put almost none).  No method arithmetic happens here.
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    q = torch.randint(0, first_hot, (N, K), generator=g, dtype=torch.int32)
    hot = torch.rand(N, K, generator=g) < frac
    q[hot] = torch.randint(first_hot, 256, (int(hot.sum()),), generator=g, dtype=torch.int32)
    return q.to(torch.uint8)


@dataclass
class LinearCase:
    config: int
    name: str
    M: int
    N: int
    K: int
    W: torch.Tensor
    X: torch.Tensor
    dY: list = field(default_factory=list)
    lambdas: tuple = (1.0, 1.0, 1.0)
    rs: tuple = (8, 4, 2)


def linear_case(config: int, name: str = "gate", with_grads: bool = True,
                M: int | None = None, shape=None) -> LinearCase:
    """One linear of configuration 1, 2, 3 or 5 with its activations and output gradients."""
    if config == 1:
        N, K = shape or (256, 256)
        tokens = 16
    else:
        shapes, tokens = mlp_shapes(config)
        N, K = shape or shapes[name]
    M = tokens if M is None else M
    W = weight(config, name, (N, K))
    X = activations(config, name, M, K)
    dY = out_grads(config, name, M, N) if with_grads else []
    return LinearCase(config, name, M, N, K, W, X, dY, LAMBDAS[config])
