"""Byte / FLOP accounting against the values the paper prints.

App. "Computation Reduction Analysis" (Eq. 13 and its table) and App. "Memory
Reduction Analysis" (Eq. 12 and its table); fixture tests/golden/paper_model_ratios.txt.
"""
import pytest

from conftest import read_golden
from paper_2410_09615_amd import accounting as A


def _rows():
    g = read_golden("paper_model_ratios.txt")
    for name, vals in g.items():
        v = vals[0]
        yield (name, int(v[0]), int(v[1]), int(v[2]), int(v[3]) / int(v[4]),
               [float(x) for x in v[5:]])


@pytest.mark.parametrize("row", list(_rows()), ids=lambda r: r[0])
def test_model_ratios_match_paper_tables(row):
    _, d, n, V, a, (f_no, f_ad, m_no, m_16, m_q4) = row
    tol = 0.0051                                   # the tables print two decimals
    assert abs(A.flop_reduction(d, n, V, a, None) - f_no) <= tol
    assert abs(A.flop_reduction(d, n, V, a, 0.1) - f_ad) <= tol
    assert abs(A.memory_ratio(d, n, V, a, None) - m_no) <= tol
    assert abs(A.memory_ratio(d, n, V, a, 0.1, adapter_bits=16) - m_16) <= tol
    assert abs(A.memory_ratio(d, n, V, a, 0.1, adapter_bits=4) - m_q4) <= tol


def test_layer_counts_sum_to_the_model_formula():
    """Summing the per-layer algorithmic FLOPs over one LLaMA-2-7B block set
    (as Eq. 13 models it: four d x d and two d x a d matrices per block, dense
    head) reproduces the paper's 1.49."""
    d, n, V, ff = 4096, 32, 32000, 11008
    r = 410                                         # 10 % of the hidden size
    m = 1
    comp = n * (4 * A.flops_alg(d, d, r, m) + A.flops_alg(ff, d, r, m) + A.flops_alg(d, ff, r, m))
    dense = n * (4 * A.flops_dense(d, d, m) + 2 * A.flops_dense(ff, d, m))
    head = 2 * d * V
    assert abs((dense + head) / (comp + head) - 1.49) <= 0.0051


def test_layer_bytes_formula():
    n, k, r, m = 4096, 4096, 410, 1
    assert A.packed_weight_bytes(n, k) == n * k * 3 // 8 + 4 * n
    assert A.layer_bytes(n, k, r, m) == 6291456 + 16384 + 2 * 410 * 8192 + 8192 + 8192
    assert A.dense_bytes(n, k, m) == 2 * n * k + 4 * 4096
    assert A.flops_eff(n, k, r, m) == 2 * n * k + 2 * r * (n + k)
    # this build's format stores 3 bits per original weight; the paper's
    # memory model counts 2 (no position metadata)
    no_meta = A.memory_ratio(4096, 32, 32000, 11008 / 4096, 0.1)
    with_meta = A.memory_ratio(4096, 32, 32000, 11008 / 4096, 0.1, metadata_bits_per_weight=1.0)
    assert with_meta > no_meta and abs(with_meta - no_meta - 0.0609) < 2e-3
