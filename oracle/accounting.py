"""Closed-form communication / memory accounting of the method (test infrastructure).

Each function restates one formula of the paper; tests pin them to the values
the paper prints (tests/golden/accounting.txt).
"""
from __future__ import annotations

import math


def bits_per_token(n_layers: int, n_groups: int, codebook_size: int, codebooks_per_layer: int = 1) -> int:
    """Sec. 2 (Grouped VQ): G * log2 K bits per token per exchange, one exchange per block."""
    return n_layers * codebooks_per_layer * n_groups * int(math.log2(codebook_size))


def full_precision_bits_per_token(n_layers: int, width: int, bits: int = 32, tensors_per_layer: int = 1) -> int:
    """Sec. 3.2: r * D bits per token per block when embeddings travel uncompressed."""
    return n_layers * tensors_per_layer * width * bits


def compression_ratio(full_bits: float, vq_bits: float) -> float:
    return full_bits / vq_bits


def fpar(tokens_per_device) -> float:
    """Appendix (heterogeneous settings), Eq. FPAR: sum_k n_k^2 / N^2."""
    n = float(sum(tokens_per_device))
    return sum(float(v) * float(v) for v in tokens_per_device) / (n * n)


def codebook_bytes(n_layers: int, codebooks_per_layer: int, codebook_size: int, width: int, elem_bytes: int) -> int:
    """Appendix (memory cost): M_codebook = L * C * K * d * b, independent of G."""
    return n_layers * codebooks_per_layer * codebook_size * width * elem_bytes


def kv_cache_bytes_original(seq_len: int, n_layers: int, width: int, elem_bytes: int) -> int:
    """Appendix (memory cost): 2 * N * L * d * b."""
    return 2 * seq_len * n_layers * width * elem_bytes


def kv_cache_bytes_astra(seq_len: int, n_layers: int, width: int, elem_bytes: int, n_devices: int,
                         n_groups: int, codebook_size: int) -> float:
    """Appendix (memory cost): local rows at full precision, non-local rows as one
    log2(K)-bit index per group."""
    local = seq_len / n_devices * n_layers * width * elem_bytes
    nonlocal_ = (n_devices - 1) * seq_len / n_devices * n_layers * n_groups * math.log2(codebook_size) / 8
    return 2 * (local + nonlocal_)
