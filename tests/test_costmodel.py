"""The FLOP model behind the benchmark's numbers reproduces the FLOP costs the paper prints (Table 2)."""
import os

import pytest

from paper_2310_12109_amd import costmodel

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table2_flop_cost.txt")


def _rows():
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            N, dense, m2 = line.split()
            yield int(N), float(dense), float(m2)


@pytest.mark.parametrize("N,dense,m2", list(_rows()))
def test_table2_flop_costs(N, dense, m2):
    # printed with 3 significant digits (the 4K dense entry is truncated rather than rounded)
    assert costmodel.paper_m2_flops(N) / 1e12 == pytest.approx(m2, abs=6e-4, rel=2e-3)
    assert costmodel.paper_dense_flops(N) / 1e12 == pytest.approx(dense, abs=1e-3, rel=5e-3)


def test_square_monarch_is_4_n_sqrt_n():
    b = 64
    assert costmodel.monarch_matmul_flops(b, b, b, b, b, b) == 4 * (b * b) * b
    # Table 2 counts two such products per column
    assert 2 * 768 * costmodel.monarch_matmul_flops(b, b, b, b, b, b) == costmodel.paper_m2_flops(b * b)


def test_conv_bytes_and_flops_config2():
    assert costmodel.conv_algorithmic_bytes(8, 768, 1024, 1024, 2) == 4 * 6144 * 1024 * 2 + 768 * 1024 * 2
    executed = costmodel.conv_executed_flops(8, 768, (64, 32))
    textbook = costmodel.conv_textbook_flops(8, 768, (64, 32))
    assert 0.25 < executed / textbook < 0.5
