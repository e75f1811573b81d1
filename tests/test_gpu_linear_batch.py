"""GPU parity of pdelta_linear_batch: several independent delta linear layers in one call.

Every layer of a batch is compared with the fp64 oracle under the tolerance rule of
parity_util.py, and bit for bit with the single-layer entry points on the same inputs when the
batched kernel and the single-layer kernel accumulate in the same order (they share the device
code of one workgroup) or the call falls back to launching layer by layer.
"""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, check_y, gpu_linear, make_case

pytestmark = pytest.mark.gpu


def build_batch(shapes, M, dtype, seed0, y_dtype):
    """[(case, axis)] and the planned batch for shapes = [(d_out, d_in, axis), ...]."""
    cases, items = [], []
    for k, (d_out, d_in, axis) in enumerate(shapes):
        L = make_case(d_out, d_in, M, dtype, "row" if axis == orc.ROW else "col", seed0 + k)
        d = L["d"]
        v = d["v_row"] if axis == orc.ROW else d["v_col"]
        cases.append((L, axis))
        items.append((d["X"], d["W_b"], d["B"], v, axis))
    plan = pd.pdelta_linear_batch_plan(items, out_dtype=y_dtype)
    return cases, plan


def check_batch(cases, plan, Ys, what, y_dtype, bit_equal_single=True):
    for k, ((L, axis), Y) in enumerate(zip(cases, Ys)):
        d = L["d"]
        v_bits = L["v_row"] if axis == orc.ROW else L["v_col"]
        ref = orc.linear(L["X"], L["W_b"], L["B"], v_bits, axis, L["dtype"])
        check_y(Y, ref, f"{what} layer {k} axis={axis}")
        if bit_equal_single:
            v = d["v_row"] if axis == orc.ROW else d["v_col"]
            single = gpu_linear(axis, d["X"], d["W_b"], d["B"], v, y_dtype)
            assert torch.equal(single.view(torch.uint8), Y.view(torch.uint8)), f"{what} layer {k}"


MIXED = [(100, 256, orc.ROW), (16, 128, orc.COL), (7, 1152, orc.COL), (256, 512, orc.ROW), (33, 384, orc.COL)]


@pytest.mark.parametrize("M", [1, 4, 16])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_batched_kernel_mixed_shapes_and_axes(M, dtype):
    for y_dtype in (torch.float32, torch.float16 if dtype == synth.F16 else torch.bfloat16):
        cases, plan = build_batch(MIXED, M, dtype, synth.seed_for(3, 500 + M), y_dtype)
        for Y in plan.Y:
            Y.fill_(float("nan"))                     # every output entry must be written
        Ys = pd.pdelta_linear_batch(plan)
        torch.cuda.synchronize()
        check_batch(cases, plan, Ys, f"batch M={M} dt={dtype} y={y_dtype}", y_dtype)


@pytest.mark.parametrize("M,shapes", [
    (17, MIXED),                                                   # M above the batched kernel's 16 tokens
    (100, MIXED[:3]),                                              # prefill path, layer by layer
    (2, [(64, 160, orc.ROW), (48, 256, orc.COL)]),                 # d_in not a multiple of 128
    (16, [(32, 4096, orc.COL), (32, 256, orc.ROW)]),               # X too large for LDS: the batched kernel reads it through L2
])
def test_layer_by_layer_fallback_gives_the_same_results(M, shapes):
    cases, plan = build_batch(shapes, M, synth.F16, synth.seed_for(3, 600 + M), torch.float32)
    Ys = pd.pdelta_linear_batch(plan)
    torch.cuda.synchronize()
    check_batch(cases, plan, Ys, f"fallback M={M}", torch.float32)


def test_one_block_of_the_7b_stack_batch1():
    # q, k, v, o, gate, up, down of one block with the benchmark's axis mix, each with its own X and Y
    shapes = [(4096, 4096, orc.ROW)] * 2 + [(4096, 4096, orc.COL)] * 2 + \
             [(11008, 4096, orc.COL), (11008, 4096, orc.ROW), (4096, 11008, orc.ROW), (4096, 11008, orc.COL)]
    cases, plan = build_batch(shapes, 1, synth.F16, synth.seed_for(3, 700), torch.float16)
    Ys = pd.pdelta_linear_batch(plan)
    torch.cuda.synchronize()
    check_batch(cases, plan, Ys, "7B block", torch.float16, bit_equal_single=False)


def test_replanning_is_not_needed_when_only_pointers_change():
    cases, plan = build_batch(MIXED[:2], 3, synth.F16, synth.seed_for(3, 800), torch.float32)
    first = [Y.clone() for Y in pd.pdelta_linear_batch(plan)]
    # point layer 0 at a fresh output buffer: edit the host array, copy it to the device again
    new_Y = torch.zeros_like(plan.Y[0])
    plan.host[0].Y = new_Y.data_ptr()
    plan.device.copy_(torch.frombuffer(bytearray(bytes(plan.host)), dtype=torch.uint8))
    plan.Y[0].zero_()
    pd.pdelta_linear_batch(plan)
    torch.cuda.synchronize()
    assert torch.equal(new_Y, first[0])
    assert torch.count_nonzero(plan.Y[0]) == 0
    assert torch.equal(plan.Y[1], first[1])


def test_empty_batch_and_empty_list():
    cases, plan = build_batch(MIXED[:2], 0, synth.F16, 5, torch.float16)
    assert [tuple(Y.shape) for Y in pd.pdelta_linear_batch(plan)] == [(0, 100), (0, 16)]
    assert pd.lib().pdelta_linear_batch(None, None, 0, 4, pd.F16, pd.F16, None) == pd.OK
