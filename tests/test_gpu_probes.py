"""The measurement build of the prefill kernel (pdelta_probe_prefill_parts): with every part of
the loop switched on it IS the product kernel, so its output must equal pdelta_linear_row's bit
for bit; every other built mask must run to completion (its output is meaningless by contract)."""
import pytest
import torch

from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,d_out,d_in", [(300, 200, 480), (512, 1024, 1056), (2048, 4096, 4096)])
def test_all_parts_on_is_the_product_kernel(M, d_out, d_in, monkeypatch):
    monkeypatch.setenv("PDELTA_TUNE", "gemm_small=0,gemm_pipe=1")        # the same kernel on both sides
    L = synth.layer_device(d_out, d_in, synth.BF16, "row", synth.seed_for(2, 9100 + M), DEV)
    B, v_row, _ = pd.pdelta_pack(L["dW"], torch.zeros_like(L["dW"]))
    X = synth.x_device(M, d_in, synth.BF16, synth.seed_for(2, 9200 + M), DEV)
    for yd in (torch.float32, torch.bfloat16):
        want = pd.pdelta_linear_row(X, L["W_b"], B, v_row, out_dtype=yd)
        got = torch.full((M, d_out), float("nan"), dtype=yd, device=DEV)
        pd.pdelta_probe_prefill_parts(15, X, L["W_b"], B, v_row, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want)


def test_every_built_mask_runs():
    M, d_out, d_in = 512, 1024, 1056                                      # 16 full steps and a partial one
    L = synth.layer_device(d_out, d_in, synth.BF16, "row", synth.seed_for(2, 9300), DEV)
    B, v_row, _ = pd.pdelta_pack(L["dW"], torch.zeros_like(L["dW"]))
    X = synth.x_device(M, d_in, synth.BF16, synth.seed_for(2, 9301), DEV)
    Y = torch.empty((M, d_out), dtype=torch.bfloat16, device=DEV)
    for parts in pd.PREFILL_PARTS_BUILT:
        pd.pdelta_probe_prefill_parts(parts, X, L["W_b"], B, v_row, Y)
        torch.cuda.synchronize()
    with pytest.raises(pd.PdeltaError):
        pd.pdelta_probe_prefill_parts(5, X, L["W_b"], B, v_row, Y)       # a mask that is not built
