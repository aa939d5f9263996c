"""The passes can be captured into a HIP graph and replayed (GPU, C ABI).

With a caller-supplied workspace a call allocates nothing, records no memset and touches no
host state that a replay would miss, so a captured sequence of calls must give, on every
replay, exactly what the same calls give eagerly -- also after the inputs changed in place and
with eager work and synchronisation between the replays."""
import numpy as np
import pytest

from paper_1412_7580_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hd(lib):
    h = lib.Handle(0)
    yield h
    h.close()


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


@pytest.mark.parametrize("cfg", [dict(S=16, f=16, fo=16, h=13, w=13, kh=3, kw=3),      # smallest benchmark layer
                                 dict(S=2, f=4, fo=4, h=70, w=70, kh=5, kw=5),         # a layer the library tiles
                                 dict(S=8, f=8, fo=12, h=27, w=13, kh=5, kw=3),        # rectangular basis 28 x 14
                                 dict(S=8, f=8, fo=8, h=27, w=27, kh=5, kw=5)],        # basis 28, shared launches
                         ids=["13x13", "70x70_tiled", "27x13_rect", "27x27"])
def test_graph_replay_equals_eager(hd, lib, cfg):
    import torch
    x, w, gy = synth.conv_inputs(seed=600, **cfg)
    dx, dw, dgy = _dev(x), _dev(w), _dev(gy)
    dims = (cfg["S"], cfg["f"], cfg["fo"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])
    saved = torch.empty(hd.saved_bytes(*dims) // 4, device="cuda", dtype=torch.float32)
    ws1 = torch.empty(hd.workspace_bytes(lib.FPROP, *dims) // 4, device="cuda", dtype=torch.float32)
    ws2 = torch.empty(hd.backward_workspace_bytes(*dims) // 4, device="cuda", dtype=torch.float32)
    y = torch.empty((cfg["S"], cfg["fo"], cfg["h"] - cfg["kh"] + 1, cfg["w"] - cfg["kw"] + 1), device="cuda")
    gx, gw = torch.empty_like(dx), torch.empty_like(dw)
    args = (cfg["f"], cfg["h"], cfg["w"], cfg["kh"], cfg["kw"])

    def step():
        hd.fft_conv_fprop_save(dx, dw, saved, y=y, ws=ws1)
        hd.fft_conv_backward(dgy, saved, *args, gx=gx, gw=gw, ws=ws2)

    def eager():
        step()
        torch.cuda.synchronize()
        return y.clone(), gx.clone(), gw.clone()

    ref = eager()                       # also the warm-up: kernel attributes are set here
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        if rep == 2:                    # new inputs, in place: replays must follow them
            dx.mul_(0.5); dgy.add_(0.25)
            ref = eager()
        y.zero_(); gx.zero_(); gw.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref[0]) and torch.equal(gx, ref[1]) and torch.equal(gw, ref[2]), rep
        _ = (dx * 2).sum().item()       # eager work and a synchronisation between replays


def test_graph_replay_of_inference_paths(hd, lib):
    """fprop on weights transformed ahead, as three launches (a layer beyond the one-launch
    kernels' range; caller's workspace) and as the one-launch kernel (no workspace at all), and
    the one-launch bprop: captured once, replayed with changing inputs."""
    import torch
    cfg = dict(S=16, f=16, fo=16, h=16, w=16, kh=3, kw=3)       # basis 16: the fused kernel needs > 64 KB of LDS
    x, w, _ = synth.conv_inputs(seed=601, **cfg)
    dx, dw = _dev(x), _dev(w)
    wf = hd.fft_conv_transform_weights(dw, cfg["h"], cfg["w"])
    big = dict(S=16, f=32, fo=48, h=16, w=16, kh=3, kw=3)
    xb, wb, _ = synth.conv_inputs(seed=602, **big)
    dxb, dwb = _dev(xb), _dev(wb)
    wfb = hd.fft_conv_transform_weights(dwb, 16, 16)
    ws = torch.empty(hd.workspace_bytes(lib.FPROP, 16, 32, 48, 16, 16, 3, 3) // 4, device="cuda", dtype=torch.float32)
    y3 = torch.empty((16, 48, 14, 14), device="cuda")
    y1 = torch.empty((16, 16, 14, 14), device="cuda")
    gx1 = torch.empty_like(dx)          # the one-launch bprop, fed with the fused fprop's output

    def step():
        hd.fft_conv_fprop_weights(dxb, wfb, 48, 3, 3, y=y3, ws=ws)
        hd.fft_conv_fprop_fused(dx, wf, cfg["fo"], 3, 3, y=y1)
        hd.fft_conv_bprop_fused(y1, wf, cfg["f"], 16, 16, 3, 3, gx=gx1)

    def eager():
        step()
        torch.cuda.synchronize()
        return y3.clone(), y1.clone(), gx1.clone()

    ref = eager()                       # warm-up: kernel attributes are set outside the capture
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        if rep == 1:
            dx.mul_(-1.5); dxb.mul_(0.75)
            ref = eager()
        y3.zero_(); y1.zero_(); gx1.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y3, ref[0]) and torch.equal(y1, ref[1]) and torch.equal(gx1, ref[2]), rep
        _ = (dx + 1).sum().item()


def test_handle_workspace_never_grows_during_capture(lib):
    """A call without a caller workspace may have to grow the handle's own buffer, which means a
    synchronisation, a free and an allocation.  Under stream capture it must refuse instead
    (workspace too small) and launch nothing; once an eager call has grown the buffer, the same
    call captures and replays like any other."""
    import torch
    cfg = dict(S=8, f=8, fo=8, h=20, w=20, kh=3, kw=3)
    x, w, _ = synth.conv_inputs(seed=603, **cfg)
    dx, dw = _dev(x), _dev(w)
    y = torch.empty((8, 8, 18, 18), device="cuda")
    hd = lib.Handle(0)                  # a fresh handle: it owns no buffer yet
    try:
        warm = lib.Handle(0)
        ref = warm.fft_conv_fprop(dx, dw).clone()    # kernel attributes are set outside any capture
        warm.close()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with pytest.raises(lib.FFTConvError, match="workspace too small"):
            with torch.cuda.graph(graph):
                hd.fft_conv_fprop(dx, dw, y=y)
        torch.cuda.synchronize()
        hd.fft_conv_fprop(dx, dw, y=y)               # eager: the buffer grows here
        torch.cuda.synchronize()
        assert torch.equal(y, ref)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            hd.fft_conv_fprop(dx, dw, y=y)           # large enough now: nothing to allocate
        for _ in range(2):
            y.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, ref)
    finally:
        hd.close()
