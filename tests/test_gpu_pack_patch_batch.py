"""GPU parity of the model-wide entry points pdelta_pack_batch and pdelta_patch_batch against
the CPU oracle, bit for bit, and against the single-layer entry points."""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, f16_dev, to_dev, words_dev, words_host
from test_gpu_pack_patch import assert_pack_equal

pytestmark = pytest.mark.gpu

# ragged rows and columns around the 64/128-row and 1024-column tiles, a one-row layer, a layer
# with d_in % 128 != 0 (sign rows not 16-byte aligned), layers on both sides of the 512-row rule
SHAPES = [(256, 512), (1, 32), (33, 96), (100, 1056), (70, 2048 + 160), (515, 1024), (640, 2080), (129, 4096),
          (2100, 1184)]          # tall layer: 512-row tiles, ragged last tile


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_pack_batch_matches_oracle_and_single_layer_calls(dtype):
    hosts, pairs = [], []
    for k, (d_out, d_in) in enumerate(SHAPES):
        L = synth.layer_host(d_out, d_in, 1, dtype, "row" if k % 2 else "col", synth.seed_for(4, 300 + k),
                             zero_frac=0.05, with_wf=True)
        hosts.append(L)
        pairs.append((to_dev(L["W_f"], dtype), to_dev(L["W_b"], dtype)))
    plan = pd.pdelta_pack_batch_plan(pairs)
    for t in plan.tensors:
        t[5].fill_(0xAB)                                   # workspace contents must not matter
        t[2].fill_(-1)
    outs = pd.pdelta_pack_batch(plan)
    torch.cuda.synchronize()
    for k, (L, (B, v_row, v_col)) in enumerate(zip(hosts, outs)):
        got = (words_host(B), synth.torch_to_bits(v_row), synth.torch_to_bits(v_col))
        assert_pack_equal(got, orc.pack(L["W_f"], L["W_b"], dtype), f"batched pack job {k} {SHAPES[k]} dt={dtype}")
        Bs, vrs, vcs = pd.pdelta_pack(*pairs[k])
        torch.cuda.synchronize()
        assert torch.equal(Bs, B) and torch.equal(vrs, v_row) and torch.equal(vcs, v_col)
    # a second run over the used workspaces gives the same bits
    keep = [(B.clone(), r.clone(), c.clone()) for B, r, c in outs]
    pd.pdelta_pack_batch(plan)
    torch.cuda.synchronize()
    for (B, r, c), (B2, r2, c2) in zip(keep, plan.out):
        assert torch.equal(B, B2) and torch.equal(r, r2) and torch.equal(c, c2)


def test_pack_batch_without_scales_or_with_one_of_them():
    L = synth.layer_host(200, 1184, 1, synth.F16, "col", 78, with_wf=True)
    want = orc.pack(L["W_f"], L["W_b"])
    pair = (to_dev(L["W_f"], synth.F16), to_dev(L["W_b"], synth.F16))
    for want_row, want_col in ((False, False), (True, False), (False, True)):
        plan = pd.pdelta_pack_batch_plan([pair, pair], want_row=want_row, want_col=want_col)
        for B, v_row, v_col in pd.pdelta_pack_batch(plan):
            torch.cuda.synchronize()
            assert np.array_equal(words_host(B), want[0])
            assert (v_row is None) == (not want_row) and (v_col is None) == (not want_col)
            if want_row:
                assert np.array_equal(synth.torch_to_bits(v_row), want[1])
            if want_col:
                assert np.array_equal(synth.torch_to_bits(v_col), want[2])


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_patch_batch_matches_oracle_out_of_place_and_in_place(dtype):
    shapes = [(256, 512), (1, 32), (37, 96), (9, 2048 + 64), (130, 4096), (16, 2048), (17, 8192 + 32)]
    items, wants, hosts = [], [], []
    for k, (d_out, d_in) in enumerate(shapes):
        axis = orc.ROW if k % 2 == 0 else orc.COL
        L = synth.layer_host(d_out, d_in, 1, dtype, "row" if axis == orc.ROW else "col", synth.seed_for(0, 900 + k))
        B, v_row, v_col = orc.pack(L["dW"], np.zeros_like(L["dW"]), dtype)
        v = v_row if axis == orc.ROW else v_col
        wants.append(orc.patch_round(L["W_b"], B, v, axis, dtype))
        hosts.append(L)
        items.append((to_dev(L["W_b"], dtype), words_dev(B), f16_dev(v), axis))
    plan = pd.pdelta_patch_batch_plan(items)
    for W_out in plan.W_out:
        W_out.fill_(float("nan"))                          # every entry must be written
    outs = pd.pdelta_patch_batch(plan)
    torch.cuda.synchronize()
    for k, (out, want) in enumerate(zip(outs, wants)):
        assert np.array_equal(synth.torch_to_bits(out), want), f"batched patch layer {k} {shapes[k]}"
        assert np.array_equal(synth.torch_to_bits(items[k][0]), hosts[k]["W_b"])          # inputs untouched
        single = pd.pdelta_patch(*items[k])
        torch.cuda.synchronize()
        assert torch.equal(single.view(torch.int16), out.view(torch.int16))
    inplace = pd.pdelta_patch_batch_plan([(W_b, B, v, axis, W_b) for (W_b, B, v, axis) in items])
    pd.pdelta_patch_batch(inplace)
    torch.cuda.synchronize()
    for k, want in enumerate(wants):
        assert np.array_equal(synth.torch_to_bits(items[k][0]), want), f"in place layer {k}"


def test_patch_batch_un_patch_restores_the_base_when_nothing_was_rounded():
    # weights and scales on a coarse grid: W_b + v B is exact, so merging with -v afterwards
    # (negated scale = the bits of v with the sign flipped) gives W_b back bit for bit
    rng = np.random.default_rng(11)
    items, bases = [], []
    for d_out, d_in in ((96, 512), (40, 1056)):
        W_b = (rng.integers(-32, 32, (d_out, d_in)) / 64.0).astype(np.float16)
        v = (rng.integers(1, 8, d_out) / 256.0).astype(np.float16)
        B = rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32)
        W = to_dev(W_b.view(np.uint16), synth.F16)
        bases.append(W.clone())
        items.append((W, words_dev(B), f16_dev(v.view(np.uint16)), pd.ROW, W))
    pd.pdelta_patch_batch(pd.pdelta_patch_batch_plan(items))
    torch.cuda.synchronize()
    assert not any(torch.equal(it[0], b) for it, b in zip(items, bases))
    pd.pdelta_patch_batch(pd.pdelta_patch_batch_plan([(W, B, -v, axis, W) for (W, B, v, axis, _) in items]))
    torch.cuda.synchronize()
    for it, b in zip(items, bases):
        assert torch.equal(it[0], b)
