"""Size and traffic accounting for the MoLE lookup path (host logic, no kernels).

Parameter counts follow the paper's complexity analysis (Sec. 3.4 and Table 1):
per layer a re-parameterized MoLE offloads d*N*|V| table parameters and loads
d*N of them per token; the model-level figures of the results table (Table 3)
are those times the layer count L.  Byte counts are what one token of the fused
forward has to move when nothing is reused: its N table rows, the router input,
the shared-FFN output, the optional residual, the output row and its id.
"""
from __future__ import annotations


def params_loaded_per_token(d: int, N: int, L: int = 1) -> int:
    """Table parameters fetched for one token: d*N per layer (Table 1), times L layers (Table 3)."""
    return d * N * L


def params_offloaded(d: int, N: int, V: int, L: int = 1) -> int:
    """Table parameters kept off-chip: d*N*|V| per layer (Table 1), times L layers (Table 3)."""
    return d * N * V * L


def lut_bytes(d: int, N: int, V: int, L: int = 1, elem_bytes: int = 2) -> int:
    return params_offloaded(d, N, V, L) * elem_bytes


def lut_bytes_loaded_per_token(d: int, N: int, L: int = 1, elem_bytes: int = 2) -> int:
    return params_loaded_per_token(d, N, L) * elem_bytes


def forward_bytes_per_token(d: int, N: int, elem_bytes: int = 2, residual: bool = False) -> int:
    """Algorithmic bytes of the fused forward per (layer, token): N rows + h + shared + out
    (+ residual) in storage precision, plus the 4-byte id."""
    acts = 3 + (1 if residual else 0)
    return elem_bytes * N * d + acts * elem_bytes * d + 4


def forward_bytes_moved(T: int, U: int, d: int, N: int, elem_bytes: int = 2,
                        residual: bool = False) -> int:
    """Bytes that must move when each of the U distinct ids' rows is read once:
    U row blocks, per-token activations, and the router weight once."""
    acts = 3 + (1 if residual else 0)
    return U * elem_bytes * N * d + T * (acts * elem_bytes * d + 4) + elem_bytes * d * N


def build_flops(V: int, d: int, D: int, N: int) -> int:
    """Two GEMMs of V x d x D per expert, 2 flop per multiply-add: 4*V*d*D*N (cf. the
    4*d*D per-token FFN cost of the complexity section)."""
    return 4 * V * d * D * N


def nf_table_bytes(rows: int, N: int, d: int, bits: int, block: int, scale_bytes: int) -> int:
    """Size of an NF-quantised table (Sec. 5.5, Table 8): bits per element plus one scale per block."""
    return rows * N * (d * bits // 8 + (d // block) * scale_bytes)


def nf_forward_bytes_per_token(d: int, N: int, bits: int, block: int, scale_bytes: int, residual: bool = False) -> int:
    """Algorithmic bytes of the dequantising forward per (layer, token): packed rows and scales,
    bf16 h / shared / out (+ residual), and the 4-byte id."""
    acts = 3 + (1 if residual else 0)
    return N * (d * bits // 8 + (d // block) * scale_bytes) + acts * 2 * d + 4
