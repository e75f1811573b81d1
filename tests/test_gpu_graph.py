"""Every entry point records plain kernel nodes only, so a caller may capture it into a HIP
graph.  Each graph here is replayed several times, with eager work and synchronisations of the
program's own between the replays, and every replay must reproduce the eager result bit for bit."""
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, make_case

pytestmark = pytest.mark.gpu


def capture(fn):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                                               # warm up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def replay_and_compare(g, outputs, expected):
    for rep in range(3):
        for o in outputs:
            o.fill_(0 if o.dtype in (torch.int32, torch.uint8) else float("nan"))
        scratch = torch.randn(1 << 16, device=DEV).sum()   # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outputs, expected):
            assert torch.equal(o.view(torch.uint8), e.view(torch.uint8)), f"replay {rep}"
        del scratch


@pytest.mark.parametrize("M", [1, 16, 40, 300, 2048])
def test_linear_in_a_graph(M):
    L = make_case(384, 512, M, synth.F16, "row", 123 + M)
    d = L["d"]
    Yr = torch.empty((M, 384), dtype=torch.float16, device=DEV)
    Yc = torch.empty((M, 384), dtype=torch.float32, device=DEV)

    def run():
        pd.pdelta_linear_row(d["X"], d["W_b"], d["B"], d["v_row"], out=Yr)
        pd.pdelta_linear_col(d["X"], d["W_b"], d["B"], d["v_col"], out=Yc)

    run()
    torch.cuda.synchronize()
    expected = [Yr.clone(), Yc.clone()]
    replay_and_compare(capture(run), [Yr, Yc], expected)


def test_pack_patch_and_gradient_in_a_graph():
    Ld = synth.layer_device(300, 1184, synth.F16, "col", 77, DEV, with_wf=True)
    X = synth.x_device(200, 1184, synth.F16, 78, DEV)
    dY = synth.x_device(200, 320, synth.F16, 79, DEV)
    B = torch.empty((300, 37), dtype=torch.int32, device=DEV)
    v_row = torch.empty(300, dtype=torch.float16, device=DEV)
    v_col = torch.empty(1184, dtype=torch.float16, device=DEV)
    ws = torch.empty(pd.pdelta_pack_workspace_bytes(300, 1184), dtype=torch.uint8, device=DEV)
    W_out = torch.empty_like(Ld["W_b"])
    B320 = torch.randint(-2 ** 31, 2 ** 31 - 1, (320, 37), dtype=torch.int32, device=DEV)
    g_row = torch.empty(320, dtype=torch.float32, device=DEV)
    g_col = torch.empty(1184, dtype=torch.float32, device=DEV)
    wsg = [torch.empty(pd.pdelta_grad_v_workspace_bytes(200, 320, 1184, a), dtype=torch.uint8, device=DEV)
           for a in (pd.ROW, pd.COL)]

    def run():
        pd.pdelta_pack(Ld["W_f"], Ld["W_b"], out=(B, v_row, v_col), workspace=ws)
        pd.pdelta_patch(Ld["W_b"], B, v_col, pd.COL, out=W_out)            # consumes the pack's outputs
        pd.pdelta_grad_v(X, dY, B320, pd.ROW, out=g_row, workspace=wsg[0])
        pd.pdelta_grad_v(X, dY, B320, pd.COL, out=g_col, workspace=wsg[1])

    run()
    torch.cuda.synchronize()
    outputs = [B, v_row, v_col, W_out, g_row, g_col]
    expected = [o.clone() for o in outputs]
    replay_and_compare(capture(run), outputs, expected)


def test_batched_entry_points_in_a_graph():
    layers = []
    for k, (d_out, d_in, axis) in enumerate([(96, 256, orc.ROW), (40, 1152, orc.COL), (256, 512, orc.ROW)]):
        L = make_case(d_out, d_in, 3, synth.F16, "row" if axis == orc.ROW else "col", 900 + k)
        d = L["d"]
        layers.append((d["X"], d["W_b"], d["B"], d["v_row"] if axis == orc.ROW else d["v_col"], axis))
    lin = pd.pdelta_linear_batch_plan(layers, out_dtype=torch.float16)
    patch = pd.pdelta_patch_batch_plan([(W, B, v, axis) for (_, W, B, v, axis) in layers])
    X3 = layers[0][0]
    vset = pd.VariantSet([(layers[0][2], layers[0][3])] * 3, orc.ROW)
    Yv = torch.empty((3, 96), dtype=torch.float16, device=DEV)

    def run():
        pd.pdelta_linear_batch(lin)
        pd.pdelta_patch_batch(patch)
        pd.pdelta_linear_variants(X3, layers[0][1], vset, out=Yv)

    run()
    torch.cuda.synchronize()
    outputs = list(lin.Y) + list(patch.W_out) + [Yv]
    expected = [o.clone() for o in outputs]
    replay_and_compare(capture(run), outputs, expected)
