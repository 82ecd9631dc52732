"""Seeded synthetic workloads for the MoE dispatch/combine path.

This module only *describes* shapes and draws random inputs.  It holds none of
the method's arithmetic (no gating, no permutation, no combine), so that both
the CPU oracle's tests and the HIP path's tests can feed from it without
sharing any code of the method itself.

Recipe (identical for every workload): with ``rng = numpy.random.default_rng(seed)``
the gate logits ``[T, E]`` are drawn first as float32 standard normals, then the
activations ``[T, H]`` as float32 standard normals.  Workloads that ask for a
skewed expert load add a per-expert bias ``-s * ln(e + 1)`` (the log of an
unnormalised Zipf(s) mass, expert index = popularity rank) to the logits in
float32.  bf16 activations are the float32 draws rounded to nearest-even and are
carried on the host as ``uint16`` bit patterns (numpy has no bf16 type).

The five named workloads follow the shapes of a sparse-MoE layer under combined
expert and tensor parallelism (hidden 8192, TP 8, EP 2 is the shape of the
paper's Table 7; the others widen experts / top-k / sequence length).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

FP32 = 0
BF16 = 1


@dataclass(frozen=True)
class Workload:
    name: str
    tokens: int            # T = batch * sequence
    hidden: int            # H, elements per token row
    dtype: int             # FP32 or BF16 (activations only; logits/gates are fp32)
    experts: int           # E
    top_k: int             # k
    ep: int                # virtual expert-parallel ranks
    tp: int                # virtual tensor-parallel ranks
    slices: int            # S chunks along the sequence
    capacity_factor: float  # 0 => dropless
    renorm: int = 1        # gates renormalised over the k winners
    zipf_s: float = 0.0    # > 0 => add -s*ln(e+1) to the logits
    padded: int = 0        # 1 => capacity-padded [E][C][H] layout of the expert-major buffer
    seed: int = 0

    def __post_init__(self):
        # the C ABI carries the capacity factor as fp32: keep the fp32-representable value here, so that
        # every consumer of a workload (CPU or GPU side) is handed exactly the same number
        object.__setattr__(self, "capacity_factor", float(np.float32(self.capacity_factor)))

    @property
    def bpe(self) -> int:
        return 4 if self.dtype == FP32 else 2

    @property
    def row_bytes(self) -> int:
        return self.hidden * self.bpe

    @property
    def units(self) -> int:
        return self.slices * self.tp

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    # small case the oracle finishes instantly
    "tiny": Workload("tiny", 256, 128, FP32, 4, 2, 2, 2, 2, 0.0),
    # Mixtral-like layer: 8 experts, top-2, one expert per virtual EP rank
    "mixtral": Workload("mixtral", 8192, 4096, BF16, 8, 2, 8, 1, 4, 2.0),
    # the paper's evaluation shape (Table 7): hidden 8192, TP 8, EP 2, 8K sequence
    "2x70b": Workload("2x70b", 8192, 8192, BF16, 2, 1, 2, 8, 4, 0.0),
    # long context; slices is swept over {1, 2, 4, 8} by the callers
    "longctx": Workload("longctx", 32768, 8192, BF16, 8, 2, 8, 8, 4, 1.25),
    # fine-grained experts with a heavily skewed load and capacity drops
    "skewed": Workload("skewed", 65536, 7168, BF16, 64, 8, 8, 4, 8, 1.25, zipf_s=1.2),
}
CONFIG_ORDER = ["tiny", "mixtral", "2x70b", "longctx", "skewed"]


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns.

    Only finite inputs are produced by the generators, so NaN handling is not needed.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_logits(w: Workload, seed: int | None = None, rng=None) -> np.ndarray:
    if rng is None:
        rng = np.random.default_rng(w.seed if seed is None else seed)
    logits = rng.standard_normal((w.tokens, w.experts), dtype=np.float32)
    if w.zipf_s > 0.0:
        bias = (-w.zipf_s * np.log(np.arange(1, w.experts + 1, dtype=np.float64))).astype(np.float32)
        logits = (logits + bias[None, :]).astype(np.float32)
    return np.ascontiguousarray(logits)


def make_inputs(w: Workload, seed: int | None = None):
    """Returns (logits float32 [T,E], x) with x float32 [T,H] or uint16 bf16 bits [T,H]."""
    rng = np.random.default_rng(w.seed if seed is None else seed)
    logits = make_logits(w, rng=rng)
    x = rng.standard_normal((w.tokens, w.hidden), dtype=np.float32)
    if w.dtype == BF16:
        x = f32_to_bf16_bits(x)
    return logits, np.ascontiguousarray(x)


def make_tied_logits(w: Workload, levels: int = 3, seed: int | None = None) -> np.ndarray:
    """Logits drawn from a handful of distinct values, so that ties are everywhere.

    Used to exercise the tie-break rule of top-k selection.
    """
    rng = np.random.default_rng(w.seed if seed is None else seed)
    vals = rng.integers(0, levels, size=(w.tokens, w.experts))
    return np.ascontiguousarray((vals.astype(np.float32) - 1.0) * np.float32(0.5))


def make_gate_weights(w: Workload, seed: int | None = None) -> np.ndarray:
    """Random-init gate weights [E, H] in the workload's activation type (uint16 bf16 bits or float32),
    drawn as standard normals scaled by 1/sqrt(H) so that the logits are O(1)."""
    rng = np.random.default_rng(10_000 + (w.seed if seed is None else seed))
    wg = (rng.standard_normal((w.experts, w.hidden), dtype=np.float32) / np.float32(np.sqrt(w.hidden))).astype(np.float32)
    return f32_to_bf16_bits(wg) if w.dtype == BF16 else np.ascontiguousarray(wg)


def make_expert_weights(w: Workload, n_out: int | None = None, seed: int | None = None) -> np.ndarray:
    """Random-init weights of one linear layer per expert, [E, N, H] (a row of H inputs per output feature; N = H
    unless given), standard normals scaled by 1/sqrt(H), in the workload's activation type."""
    n_out = w.hidden if n_out is None else n_out
    rng = np.random.default_rng(20_000 + (w.seed if seed is None else seed))
    we = rng.standard_normal((w.experts, n_out, w.hidden), dtype=np.float32)
    we *= np.float32(1.0 / np.sqrt(w.hidden))
    return f32_to_bf16_bits(we) if w.dtype == BF16 else np.ascontiguousarray(we)
