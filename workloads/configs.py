"""Named decode workloads and the byte/flop model that the roofline report uses.

Holds shapes and counting formulas only: no arithmetic of the decode step
itself lives here, so both the HIP path's tests and the CPU oracle's tests may
import it.

Notation follows the paper (Section 2.2): d_model (E), d_ff (F), n_heads (H),
batch B; d_head and the context capacity L_ctx are added.  One decode step
streams every weight and every live KV-cache entry from HBM once (Section 2,
"Memory costs"), which is what `algorithmic_bytes` counts.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

MASTER_SEED = 221105102


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    d_ff: int
    batch: int
    l_ctx: int
    # positions recipe: "full" -> every sequence decodes slot l_ctx-1;
    # "ragged" -> uniform integers in [pos_lo, pos_hi)
    positions: str = "full"
    pos_lo: int = 0
    pos_hi: int = 0
    rope_base: float = 10000.0
    ln_eps: float = 1e-6
    n_kv_heads: int = 1
    # storage of the two projection matrices: "int8" (with per-channel bf16 scales,
    # Section 3.6) or "bf16" (no scales: the baseline of Section 4.4)
    weights: str = "int8"

    @property
    def n_in(self) -> int:
        """Columns of the fused input projection: q | k | v | gate | up (k and v have one
        block of d_head columns per K/V head)."""
        return self.n_heads * self.d_head + 2 * self.n_kv_heads * self.d_head + 2 * self.d_ff

    @property
    def k_out(self) -> int:
        """Rows of the fused output projection: attention out | FFN activation."""
        return self.n_heads * self.d_head + self.d_ff

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # tiny single layer; the oracle runs it in milliseconds
    "c1_tiny": Workload("c1_tiny", 1, 256, 4, 64, 1024, 1, 128),
    # PaLM-8B-shaped
    "c2_8b": Workload("c2_8b", 32, 4096, 16, 256, 16384, 8, 2048),
    # PaLM-62B-shaped, the configuration the bandwidth target is quoted on
    "c3_62b": Workload("c3_62b", 64, 8192, 32, 256, 32768, 64, 2048),
    # one of eight 1D weight-stationary shards of a PaLM-540B-shaped stack
    # (Section 3.2.1): 6 of 48 heads, 9216 of 73728 FFN columns, K/V head replicated
    "c4_540b_shard8": Workload("c4_540b_shard8", 118, 18432, 6, 256, 9216, 32, 2048),
    # long-context, KV-bound regime (Section 4.2)
    "c5_62b_long": Workload("c5_62b_long", 64, 8192, 32, 256, 32768, 256, 8192,
                            positions="ragged", pos_lo=4096, pos_hi=8192),
}

# Variants for the comparisons of Section 4.2 / Section 4.4 (not among the five named workloads): the
# multihead twin of the 62B-shaped stack (one K/V head per query head, d_head 128 as in the
# paper's multihead variant) and the multiquery stack at the batch that twin fits at.
VARIANTS: Dict[str, Workload] = {
    "c3_62b_b32": Workload("c3_62b_b32", 64, 8192, 32, 256, 32768, 32, 2048),
    "c3_62b_b32_multihead": Workload("c3_62b_b32_multihead", 64, 8192, 64, 128, 32768, 32, 2048, n_kv_heads=64),
    # the 62B-shaped stack with bf16 weights (Section 4.4 compares the two weight formats)
    "c3_62b_bf16w": Workload("c3_62b_bf16w", 64, 8192, 32, 256, 32768, 64, 2048, weights="bf16"),
}


def weight_bytes_per_layer(w: Workload) -> int:
    """Bytes of the two fused projection matrices of one layer (one per int8 weight, two per
    bf16 weight)."""
    return (w.d_model * w.n_in + w.k_out * w.d_model) * (2 if w.weights == "bf16" else 1)


def weight_bytes(w: Workload) -> int:
    return w.n_layers * weight_bytes_per_layer(w)


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, d_head: int, bytes_per_el: int = 2) -> int:
    """K and V of one token of one sequence over the whole stack."""
    return 2 * n_layers * n_kv_heads * d_head * bytes_per_el


def kv_read_bytes(w: Workload, positions: List[int]) -> int:
    """KV bytes one decode step reads: slots 0..P_b inclusive for every sequence."""
    tokens = sum(int(p) + 1 for p in positions)
    return kv_bytes_per_token(w.n_layers, w.n_kv_heads, w.d_head) * tokens


def kv_alloc_bytes(w: Workload) -> int:
    return kv_bytes_per_token(w.n_layers, w.n_kv_heads, w.d_head) * w.batch * w.l_ctx


def algorithmic_bytes(w: Workload, positions: List[int]) -> int:
    """HBM bytes a decode step must move: int8 weights + KV cache read."""
    return weight_bytes(w) + kv_read_bytes(w, positions)


def algorithmic_flops(w: Workload, positions: List[int]) -> int:
    """2 flops per (token, parameter) pair (Section 2, "Compute costs") plus the
    attention contractions (q.K and p.V over every live slot and head)."""
    tokens = sum(int(p) + 1 for p in positions)
    return (2 * weight_bytes(w) * w.batch
            + 4 * w.n_layers * w.n_heads * w.d_head * tokens)


def max_context_tokens(hbm_bytes_total: float, kv_fraction: float, n_layers: int,
                       kv_heads_resident: int, d_head: int, batch: int) -> float:
    """Longest context whose KV cache fits in `kv_fraction` of the HBM of a
    slice (Table 1).  `kv_heads_resident` counts K/V head copies held across
    the whole slice for one sequence."""
    per_tok = kv_bytes_per_token(n_layers, kv_heads_resident, d_head)
    return hbm_bytes_total * kv_fraction / (per_tok * batch)
