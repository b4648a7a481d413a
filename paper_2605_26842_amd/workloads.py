"""Seeded synthetic workloads: matrix shape lists and input generators.

This module holds no optimizer arithmetic.  It only names the parameter sets
the benchmarks and tests run on and draws the random inputs (initial weights
and a correlated-Gaussian gradient stream) that both the CPU oracle and the
HIP path consume.  The real workload of the paper is the gradient stream of
MoE language-model pre-training (Sec. 6, model descriptions); those runs need
private data, so seeded synthetic inputs of the same shapes stand in.

Recipe
------
* weights      W   ~ N(0, 0.02^2), cast to the parameter dtype
* gradients    g_1 = sigma * z_1
               g_k = rho * g_{k-1} + sqrt(1 - rho^2) * sigma * z_k,  z_k ~ N(0, 1) iid
  with sigma = 1e-3 and rho = 0.9 (a stationary AR(1) stream, so consecutive
  gradients differ by a non-trivial amount and the acceleration buffer is
  exercised).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Iterator, List, Optional, Sequence, Tuple

import torch

GRAD_SIGMA = 1e-3
GRAD_RHO = 0.9
WEIGHT_STD = 0.02
BASE_SEED = 0x4D4F4E41  # "MONA"


@dataclass(frozen=True)
class MatrixSpec:
    """`count` weight matrices of shape m x n sharing a name prefix."""
    name: str
    m: int
    n: int
    count: int = 1


@dataclass(frozen=True)
class Workload:
    name: str
    specs: Tuple[MatrixSpec, ...]
    w_dtype: torch.dtype
    steps: int
    note: str = ""

    def shapes(self) -> List[Tuple[int, int]]:
        out: List[Tuple[int, int]] = []
        for s in self.specs:
            out.extend([(s.m, s.n)] * s.count)
        return out

    def names(self) -> List[str]:
        out: List[str] = []
        for s in self.specs:
            if s.count == 1:
                out.append(s.name)
            else:
                out.extend(f"{s.name}[{i}]" for i in range(s.count))
        return out

    def num_elements(self) -> int:
        return sum(s.m * s.n * s.count for s in self.specs)

    def ns_flops_dense(self, ns_steps: int = 5) -> float:
        """Dense-equivalent Newton-Schulz flop count, T * (4 p^2 q + 2 p^3)."""
        f = 0.0
        for s in self.specs:
            p, q = min(s.m, s.n), max(s.m, s.n)
            f += s.count * ns_steps * (4.0 * p * p * q + 2.0 * p ** 3)
        return f

    def ns_flops_symmetric(self, ns_steps: int = 5) -> float:
        """Flop count when the two symmetric products are taken on one triangle:
        T * (3 p^2 q + p^3)."""
        f = 0.0
        for s in self.specs:
            p, q = min(s.m, s.n), max(s.m, s.n)
            f += s.count * ns_steps * (3.0 * p * p * q + 1.0 * p ** 3)
        return f


def _moe_layer(hidden: int, ffn: int, experts: int, router: bool) -> Tuple[MatrixSpec, ...]:
    specs = [
        MatrixSpec("attn.wq", hidden, hidden),
        MatrixSpec("attn.wk", hidden, hidden),
        MatrixSpec("attn.wv", hidden, hidden),
        MatrixSpec("attn.wo", hidden, hidden),
        MatrixSpec("expert.up", hidden, ffn, experts),
        MatrixSpec("expert.gate", hidden, ffn, experts),
        MatrixSpec("expert.down", ffn, hidden, experts),
    ]
    if router:
        specs += [MatrixSpec("proj.tall", hidden, 512), MatrixSpec("proj.wide", 512, hidden)]
    return tuple(specs)


def _repeat_layers(layer: Sequence[MatrixSpec], layers: int) -> Tuple[MatrixSpec, ...]:
    out = []
    for li in range(layers):
        out.extend(MatrixSpec(f"L{li}.{s.name}", s.m, s.n, s.count) for s in layer)
    return tuple(out)


WORKLOADS = {
    # configs[0]: one fp32 matrix, the case the oracle finishes in well under a second
    "single_256x512": Workload(
        "single_256x512", (MatrixSpec("w", 256, 512),), torch.float32, 3,
        "single fp32 weight matrix, 3 steps"),
    # configs[1]: one dense transformer block, hidden 2048
    "dense_block_h2048": Workload(
        "dense_block_h2048",
        (MatrixSpec("attn.wq", 2048, 2048), MatrixSpec("attn.wk", 2048, 2048),
         MatrixSpec("attn.wv", 2048, 2048), MatrixSpec("attn.wo", 2048, 2048),
         MatrixSpec("ffn.up", 2048, 8192), MatrixSpec("ffn.down", 8192, 2048)),
        torch.bfloat16, 10, "attention + FFN pair of one dense block"),
    # configs[2]: MoE expert bank, 64 experts
    "moe_bank_e64": Workload(
        "moe_bank_e64",
        (MatrixSpec("expert.up", 2048, 1024, 64), MatrixSpec("expert.gate", 2048, 1024, 64),
         MatrixSpec("expert.down", 1024, 2048, 64)),
        torch.bfloat16, 10, "64 experts x (up, gate, down)"),
    # configs[3]: one large MoE layer, hidden 4096, 128 experts
    "moe_layer_h4096_e128": Workload(
        "moe_layer_h4096_e128", _moe_layer(4096, 1536, 128, router=False),
        torch.bfloat16, 5, "attention 4096x4096 x4 + 128 experts x (up, gate, down)"),
    # configs[4]: 24 such layers plus router/projection matrices.  At 18 bytes of
    # resident data per element it is ~1.07 TB and does not fit one GPU; the
    # resident subset below (`moe_stack_l4`) is what one GPU can show.
    "moe_stack_l24": Workload(
        "moe_stack_l24", _repeat_layers(_moe_layer(4096, 1536, 128, router=True), 24),
        torch.bfloat16, 3, "24 MoE layers (exceeds one GPU's memory)"),
    "moe_stack_l4": Workload(
        "moe_stack_l4", _repeat_layers(_moe_layer(4096, 1536, 128, router=True), 4),
        torch.bfloat16, 3, "4 resident layers of the 24-layer stack"),
    # ragged shapes for parity tests: not multiples of any tile, tall/wide/square, tiny
    "ragged_mix": Workload(
        "ragged_mix",
        (MatrixSpec("r.wide", 100, 300), MatrixSpec("r.tall", 333, 130),
         MatrixSpec("r.square", 257, 257), MatrixSpec("r.tiny", 3, 5),
         MatrixSpec("r.row", 1, 64), MatrixSpec("r.col", 70, 1),
         MatrixSpec("r.group", 192, 136, 3)),
        torch.float32, 3, "ragged shapes for edge-case parity"),
    # the paper's own expert shapes (Sec. 6 model descriptions), supplementary
    "paper_moe_1b": Workload(
        "paper_moe_1b",
        (MatrixSpec("expert.up", 768, 256, 128), MatrixSpec("expert.down", 256, 768, 128)),
        torch.bfloat16, 5, "MOE-1B-A0d2B expert shapes"),
    "paper_moe_6b": Workload(
        "paper_moe_6b",
        (MatrixSpec("expert.up", 1536, 1024, 128), MatrixSpec("expert.down", 1024, 1536, 128)),
        torch.bfloat16, 5, "MOE-6B-A0d5B expert shapes"),
    "paper_moe_68b": Workload(
        "paper_moe_68b",
        (MatrixSpec("expert.up", 3072, 1024, 256), MatrixSpec("expert.down", 1024, 3072, 256)),
        torch.bfloat16, 5, "MOE-68B-A3B expert shapes (one layer: hidden 3072, 256 experts of FFN size 1024)"),
}

# order of BASELINE configs
CONFIG_ORDER = ("single_256x512", "dense_block_h2048", "moe_bank_e64",
                "moe_layer_h4096_e128", "moe_stack_l24")


@dataclass
class HParams:
    """Hyper-parameters of the step (Alg. 1, REQUIRE line); defaults follow the
    benchmark recipe: alpha from the rule alpha = -1 / (2 (1 - beta_a))."""
    lr: float = 2e-2
    momentum: float = 0.95
    beta_a: float = 0.9
    alpha: float = -5.0
    weight_decay: float = 0.1
    ns_steps: int = 5
    ns_a: float = 3.4445
    ns_b: float = -4.7750
    ns_c: float = 2.0315
    ns_eps: float = 0.0
    gamma_coeff: float = 0.2
    ns_precision: int = 0
    flags: int = 0


def matrix_seed(workload_index: int, matrix_index: int) -> int:
    return BASE_SEED + 1000003 * workload_index + matrix_index


def _generator(seed: int, device: torch.device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def draw_weight(shape: Tuple[int, int], seed: int, dtype: torch.dtype,
                device: torch.device | str = "cpu") -> torch.Tensor:
    device = torch.device(device)
    gen = _generator(seed ^ 0x5EED0001, device)
    w = torch.empty(shape, dtype=torch.float32, device=device)
    w.normal_(0.0, WEIGHT_STD, generator=gen)
    return w.to(dtype)


class GradientStream:
    """Stationary AR(1) Gaussian gradient stream for one matrix (fp32)."""

    def __init__(self, shape: Tuple[int, int], seed: int,
                 device: torch.device | str = "cpu",
                 sigma: float = GRAD_SIGMA, rho: float = GRAD_RHO):
        self.shape = tuple(shape)
        self.device = torch.device(device)
        self.gen = _generator(seed ^ 0x6AD00002, self.device)
        self.sigma = float(sigma)
        self.rho = float(rho)
        self.prev: Optional[torch.Tensor] = None

    def next(self, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        z = torch.empty(self.shape, dtype=torch.float32, device=self.device)
        z.normal_(0.0, 1.0, generator=self.gen)
        if self.prev is None:
            g = z.mul_(self.sigma)
        else:
            g = z.mul_(math.sqrt(1.0 - self.rho * self.rho) * self.sigma).add_(self.prev, alpha=self.rho)
        self.prev = g
        if out is not None:
            out.copy_(g)
            return out
        return g.clone()


    def advance(self, g: torch.Tensor) -> torch.Tensor:
        """The next gradient written over the previous one: `g` must be the tensor the last call
        returned or filled (any fp32 tensor of the stream's shape at the first call).  For workloads
        whose gradients are too large to keep twice.  Draws the same z_k as `next`; the AR(1)
        combination is rounded in a different order, so use one of the two consistently."""
        z = torch.empty(self.shape, dtype=torch.float32, device=self.device)
        z.normal_(0.0, 1.0, generator=self.gen)
        if self.prev is None:
            g.copy_(z.mul_(self.sigma))
        else:
            g.mul_(self.rho).add_(z, alpha=math.sqrt(1.0 - self.rho * self.rho) * self.sigma)
        self.prev = g
        return g


def make_inputs(workload: Workload, workload_index: int = 0,
                device: torch.device | str = "cpu",
                steps: Optional[int] = None,
                g_dtype: torch.dtype = torch.float32):
    """Draw initial weights and `steps` gradients for every matrix.

    Returns (weights, grads) with weights[i] a tensor of the workload's
    parameter dtype and grads[k][i] the k-th gradient of matrix i.
    Intended for sizes that fit comfortably in memory `steps` times over.
    """
    steps = workload.steps if steps is None else steps
    shapes = workload.shapes()
    weights = [draw_weight(s, matrix_seed(workload_index, i), workload.w_dtype, device)
               for i, s in enumerate(shapes)]
    streams = [GradientStream(s, matrix_seed(workload_index, i), device)
               for i, s in enumerate(shapes)]
    grads = [[st.next().to(g_dtype) for st in streams] for _ in range(steps)]
    return weights, grads


# Non-matrix parameters of a model of the benchmark's size (Sec. 4.1: embeddings, biases and norm
# gains are stepped by AdamW): an input embedding and an output head of 131072 x 4096 and the norm
# gains of 24 layers.  bf16 parameters, fp32 gradients.
VECTOR_WORKLOADS = {
    "embeddings_h4096_v128k": tuple([(131072, 4096)] * 2 + [(4096,)] * 49),
    "small_vectors": tuple([(4096,)] * 49 + [(1000,), (3,)]),
}


def draw_vector_inputs(shapes, seed: int, w_dtype: torch.dtype, g_dtype: torch.dtype, device, steps: int = 1):
    """Seeded parameters N(0, 0.02^2) and `steps` gradient sets N(0, sigma^2) for tensors of any shape."""
    gen = torch.Generator(device=device).manual_seed(BASE_SEED + 7919 * seed)
    params = [(torch.randn(s, generator=gen, device=device) * WEIGHT_STD).to(w_dtype) for s in shapes]
    grads = [[(torch.randn(s, generator=gen, device=device) * GRAD_SIGMA).to(g_dtype) for s in shapes]
             for _ in range(steps)]
    return params, grads
