"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation,
no memset nodes), so a whole layer step can be captured in a HIP graph and replayed: every replay must
reproduce the eager result bit for bit, with eager work and synchronisations between the replays."""
import pytest
import torch

from paper_2602_16986_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,bias_grad", [("bf16-sparse", False), ("bf16-targets", True)])
def test_layer_step_replays_from_a_graph(name, bias_grad):
    from paper_2602_16986_amd.runner import DeviceWorkload
    w = wl.small(name)
    dw = DeviceWorkload(w, bias_grad=bias_grad)
    outs = [dw.out, dw.y, dw.dattn, dw.du, dw.dgamma, dw.dq, dw.dk, dw.dv] + ([dw.dtable] if bias_grad else [])
    dw.layer_step()                                   # eager: also sets the kernels' attributes once
    torch.cuda.synchronize()
    if bias_grad:
        # the per-distance sums of the bias gradient are added with atomics: equal up to rounding order
        ref_table = dw.dtable.clone()
        outs = outs[:-1]
    ref = [t.clone() for t in outs]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            dw.layer_step()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in outs:
            t.fill_(float("nan")) if t.is_floating_point() else t.zero_()
        scratch = torch.randn(1 << 16, device=dw.device).sum()      # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, ref):
            assert torch.equal(got, want), f"replay {replay} differs from the eager step"
        if bias_grad:
            torch.testing.assert_close(dw.dtable, ref_table, rtol=1e-4, atol=1e-6)
        del scratch


def _capture_and_replay(fn, outs, device):
    fn()                                              # eager: kernel attributes, GEMM plans
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in outs:
            t.fill_(float("nan"))
        scratch = torch.randn(1 << 16, device=device).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, ref):
            assert torch.equal(got, want), f"replay {replay} differs from the eager call"
        del scratch


def test_fp8_layer_forward_replays_from_a_graph():
    """The FP8 forward of the layer runs on this library's kernels only (norm + quantisation, FP8 GEMMs, attention):
    captured after one eager call, it replays bit-identically."""
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-sparse-targets"), fp8=True)
    _capture_and_replay(dl.fwd, [dl.out, dl.u_saved, dl.attn_saved, dl.mean, dl.rstd], dl.device)


def test_bf16_layer_step_replays_from_a_graph():
    """Forward and backward of the bf16 layer, GEMM library calls included: the plans are made by the eager call, the
    captured calls only enqueue."""
    from paper_2602_16986_amd.runner import DeviceLayer
    dl = DeviceLayer(wl.layer_case("layer-small-sparse-targets"))
    _capture_and_replay(dl.step, [dl.out, dl.dz, dl.d_norm_w, dl.d_w1, dl.d_gated_norm_w, dl.d_w2], dl.device)
