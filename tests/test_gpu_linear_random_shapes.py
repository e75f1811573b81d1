"""Seeded random shapes through every dispatch branch of pdelta_linear_row / pdelta_linear_col
(staged and plain decode kernels, 8 and 16 waves, X staged or not, small-tile / two-per-CU /
pipelined prefill), each compared with the fp64 oracle under the rule of parity_util.py."""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import synth
from parity_util import check_y, gpu_linear, make_case

pytestmark = pytest.mark.gpu


def random_configs(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        d_in = 32 * int(rng.choice([1, 2, 3, 4, 5, 8, 16, 31, 32, 33, 64, 100, 128, 200, 256, 257, 300]))
        d_out = int(rng.choice([1, 7, 16, 17, 40, 64, 100, 129, 256, 300, 500]))
        M = int(rng.choice([1, 2, 3, 5, 6, 7, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 128, 129, 200, 256, 257, 400]))
        if M * d_out * d_in > 1.5e8:
            continue
        out.append((M, d_out, d_in, int(rng.integers(0, 2)), int(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("M,d_out,d_in,dtype,sigma_col", random_configs(48, 20251219))
def test_random_shape(M, d_out, d_in, dtype, sigma_col):
    L = make_case(d_out, d_in, M, dtype, "col" if sigma_col else "row", 1000 * M + d_out + d_in)
    d = L["d"]
    for axis, v_bits, v_dev in ((orc.ROW, L["v_row"], d["v_row"]), (orc.COL, L["v_col"], d["v_col"])):
        ref = orc.linear(L["X"], L["W_b"], L["B"], v_bits, axis, L["dtype"])
        Y = gpu_linear(axis, d["X"], d["W_b"], d["B"], v_dev, torch.float32)
        check_y(Y, ref, f"random M={M} {d_out}x{d_in} dt={dtype} axis={axis}")
