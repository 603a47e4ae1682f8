"""Algorithmic byte and FLOP counts of the compressed layer and of a model.

Per layer (N = d_out, K = d_in, r = adapter rank, M = tokens), what the method
has to move and compute, not the dense work it avoids:

  bytes      = N K / 4 (two int4 codes per group of 4 inputs)
             + N K / 8 (two 2-bit positions per group)
             + 4 N     (fp32 scale per output row)
             + 2 r (N + K) (fp16 adapters, true rank; 4-bit adapters: r (N + K) / 2 + fp16 group scales)
             + 2 M K + 2 M N (fp16 X in, fp16 Y out)
  flops_alg  = 2 M N K / 2 + 2 M r (N + K)   (2:4 halves the weight term and
               quantization saves none: paper, App. "Computation Reduction
               Analysis")
  flops_eff  = 2 M N K + 2 M r (N + K)       (dense-equivalent)

Model level: the paper's memory and FLOP ratios (App. "Memory Reduction
Analysis" Eq. 12 and App. "Computation Reduction Analysis" Eq. 13) for a
transformer with hidden size d, n blocks, vocabulary V and up/down ratio a.
Eq. 12 as printed carries no bit widths; the table under it is reproduced by
weighting each term with its storage width (16-bit dense, 4-bit codes on the
kept half, 16- or 4-bit adapters), which is what `memory_ratio` does.
"""
from __future__ import annotations


def packed_weight_bytes(n: int, k: int) -> int:
    return n * k // 4 + n * k // 8 + 4 * n


def adapter_bytes(n: int, k: int, r: int) -> int:
    return 2 * r * (n + k)


def adapter_bytes_q4(n: int, k: int, r: int) -> int:
    """4-bit group-128 adapters (paper, Sec. 3.3): half a byte per element plus one
    fp16 scale per group of 128 elements of a row of L [n][r] or R [r][k]."""
    return (r * (n + k) + 1) // 2 + 2 * (n * ((r + 127) // 128) + r * ((k + 127) // 128))


def layer_bytes(n: int, k: int, r: int, m: int, adapter_bits: int = 16) -> int:
    ad = adapter_bytes_q4(n, k, r) if adapter_bits == 4 else adapter_bytes(n, k, r)
    return packed_weight_bytes(n, k) + ad + 2 * m * k + 2 * m * n


def dense_bytes(n: int, k: int, m: int) -> int:
    return 2 * n * k + 2 * m * k + 2 * m * n


def flops_alg(n: int, k: int, r: int, m: int) -> int:
    return m * n * k + 2 * m * r * (n + k)


def flops_eff(n: int, k: int, r: int, m: int) -> int:
    return 2 * m * n * k + 2 * m * r * (n + k)


def flops_dense(n: int, k: int, m: int) -> int:
    return 2 * m * n * k


def pack_bytes(n: int, k: int) -> int:
    """slim_pack: fp32 W in, packed codes + metadata + scales out."""
    return 4 * n * k + packed_weight_bytes(n, k)


def flop_reduction(d: int, n_blocks: int, vocab: int, a: float, r: float | None,
                   sparsity: float = 0.5) -> float:
    """Eq. 13: dense FLOPs / compressed FLOPs per token.  Per block: four d x d
    attention projections and two d x a d feed-forward matrices; the kept
    fraction (1 - sparsity) of each; adapters of rank r d on each (r None =
    no adapters); the d x V head is left dense."""
    keep = 1.0 - sparsity
    dense = n_blocks * (4 * d * d + 2 * d * d * a) + d * vocab
    comp = n_blocks * (4 * d * d * keep + 2 * d * d * a * keep) + d * vocab
    if r is not None:
        comp += n_blocks * (4 * 2 * d * d * r + 2 * (d * d * r + d * d * r * a))
    return dense / comp


def memory_ratio(d: int, n_blocks: int, vocab: int, a: float, r: float | None,
                 weight_bits: int = 4, adapter_bits: int = 16, sparsity: float = 0.5,
                 dense_bits: int = 16, metadata_bits_per_weight: float = 0.0) -> float:
    """Eq. 12 with storage widths: compressed size / dense size.  The paper's
    table counts weight_bits on the kept half and no 2:4 position metadata;
    pass metadata_bits_per_weight=1.0 for this build's format (two 2-bit
    positions per group of 4 = 1 bit per original weight)."""
    keep = 1.0 - sparsity
    block_params = 4 * d * d + 2 * d * d * a
    dense = (n_blocks * block_params + d * vocab) * dense_bits
    comp = n_blocks * block_params * (keep * weight_bits + metadata_bits_per_weight)
    comp += d * vocab * dense_bits
    if r is not None:
        adapter_params = 4 * 2 * d * d * r + 2 * (d * d * r + d * d * r * a)
        comp += n_blocks * adapter_params * adapter_bits
    return comp / dense
