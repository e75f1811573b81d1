"""Seeded random shapes for pdelta_pack and pdelta_patch (single-layer and batched), bit for bit
against the oracle: ragged rows and columns around the 64/128/512-row and 1024/2048-column
tiles of the kernels."""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, f16_dev, to_dev, words_dev, words_host
from test_gpu_pack_patch import assert_pack_equal

pytestmark = pytest.mark.gpu


def random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    return [(int(rng.choice([1, 5, 31, 32, 33, 63, 64, 65, 127, 129, 200, 511, 513, 700, 2049])),
             32 * int(rng.choice([1, 2, 3, 4, 5, 16, 31, 32, 33, 63, 64, 65, 100])),
             int(rng.integers(0, 2))) for _ in range(n)]


SHAPES = random_shapes(20, 19720)


def test_random_shapes_pack_and_patch_single_and_batched():
    for dtype in (synth.F16, synth.BF16):
        hosts, pairs, wants = [], [], []
        for k, (d_out, d_in, col) in enumerate(SHAPES):
            L = synth.layer_host(d_out, d_in, 1, dtype, "col" if col else "row", 5000 + k, zero_frac=0.05, with_wf=True)
            hosts.append(L)
            pairs.append((to_dev(L["W_f"], dtype), to_dev(L["W_b"], dtype)))
            wants.append(orc.pack(L["W_f"], L["W_b"], dtype))
        plan = pd.pdelta_pack_batch_plan(pairs)
        outs = pd.pdelta_pack_batch(plan)
        torch.cuda.synchronize()
        items, patched = [], []
        for k, (want, (B, v_row, v_col)) in enumerate(zip(wants, outs)):
            what = f"shape {SHAPES[k]} dt={dtype}"
            assert_pack_equal((words_host(B), synth.torch_to_bits(v_row), synth.torch_to_bits(v_col)), want, "batched " + what)
            Bs, vrs, vcs = pd.pdelta_pack(*pairs[k])
            torch.cuda.synchronize()
            assert_pack_equal((words_host(Bs), synth.torch_to_bits(vrs), synth.torch_to_bits(vcs)), want, "single " + what)
            axis = orc.COL if SHAPES[k][2] else orc.ROW
            v_bits = want[2] if axis == orc.COL else want[1]
            patched.append(orc.patch_round(hosts[k]["W_b"], want[0], v_bits, axis, dtype))
            items.append((pairs[k][1], words_dev(want[0]), f16_dev(v_bits), axis))
            single = pd.pdelta_patch(*items[-1])
            torch.cuda.synchronize()
            assert np.array_equal(synth.torch_to_bits(single), patched[-1]), "patch " + what
        for k, out in enumerate(pd.pdelta_patch_batch(pd.pdelta_patch_batch_plan(items))):
            torch.cuda.synchronize()
            assert np.array_equal(synth.torch_to_bits(out), patched[k]), f"batched patch shape {SHAPES[k]} dt={dtype}"
