"""Table 1's MSE and misalignment columns recomputed from the oracle's quantizers (no GPU).

The misalignment column pins something the MSE column does not: the sign and size of the magnitude
bias of each rounding scheme (zero for stochastic rounding, about 1 % for the two nearest-rounding
schemes), as Section 4.3 defines it through the rescaling factor S."""
import os

import pytest

from indep import GOLDEN, read_table1
from oracle import table1


def read_misalignment():
    out = {}
    with open(os.path.join(GOLDEN, "table1_misalignment.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, paper, lo, hi = line.split()
            out[name] = (float(paper), float(lo), float(hi))
    return out


@pytest.fixture(scope="module")
def columns():
    return table1.table1(rows=384, k=2048, seed=3, block=32, sr_seeds=6)


@pytest.mark.parametrize("scheme", ["sr_absmax", "rtn_absmax", "quest"])
def test_mse_column(columns, scheme):
    paper, lo, hi = read_table1()[scheme]
    assert lo <= columns[scheme][0] <= hi, columns[scheme]


@pytest.mark.parametrize("scheme", ["sr_absmax", "rtn_absmax", "quest"])
def test_misalignment_column(columns, scheme):
    paper, lo, hi = read_misalignment()[scheme]
    assert lo <= columns[scheme][1] <= hi, columns[scheme]


def test_ordering_of_the_schemes(columns):
    # the trade-off the table illustrates: SR has the largest error and no bias, RTN AbsMax less error
    # and some bias, QuEST the least error and the most bias
    mse = {k: v[0] for k, v in columns.items()}
    mis = {k: v[1] for k, v in columns.items()}
    assert mse["sr_absmax"] > mse["rtn_absmax"] > mse["quest"]
    assert abs(mis["sr_absmax"]) < mis["rtn_absmax"] < mis["quest"]


def test_wider_blocks_keep_the_columns():
    # a rotation of Gaussian data is Gaussian data: the columns do not depend on the Hadamard block
    res = table1.table1(rows=128, k=2048, seed=4, block=256, sr_seeds=2)
    for scheme, (paper, lo, hi) in read_table1().items():
        assert lo <= res[scheme][0] <= hi, (scheme, res[scheme])
