"""The allocation-free forward entry point (switchback_forward_static) against switchback_forward, through the C ABI:
same kernels, so every output must match bit for bit.  Two calls in a row share the library's per-GPU scratch array;
the second is a smaller layer, so stale partial maxima of the first call would show up as a wrong weight scale."""
import numpy as np
import pytest
import torch

from paper_2304_13013_amd import switchback as sb

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def draw(gen, shape, scale):
    return (torch.randn(shape, generator=gen, device=DEV, dtype=torch.float32) * scale).to(torch.bfloat16)


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def test_forward_static_matches_forward_on_two_calls_in_a_row():
    gen = torch.Generator(device=DEV)
    gen.manual_seed(71)
    # first a layer whose tensor-wise first pass fills many partial maxima and whose weights are LARGE, then a smaller
    # layer with small weights: a partial maximum left over from the first call would dominate the second's absmax
    for (b, n, m, wscale) in ((1500, 1280, 2304, 3.0), (333, 256, 192, 0.02)):
        x, w = draw(gen, (b, n), 1.0), draw(gen, (m, n), wscale)
        ref_bufs, bufs = sb.LayerBuffers(b, n, m, DEV), sb.LayerBuffers(b, n, m, DEV)
        for dtype in (torch.bfloat16, torch.float32, torch.int32):
            y_ref, _ = sb.forward(x, w, bufs=ref_bufs, y_dtype=dtype)
            y = torch.empty_like(y_ref)
            before = torch.cuda.memory_allocated()
            sb.forward_static(x, w, bufs, y=y, y_dtype=dtype)
            assert torch.cuda.memory_allocated() == before          # the binding allocated nothing either
            torch.cuda.synchronize()
            assert same_bits(y, y_ref), "output differs (%s)" % dtype
            for name in ("xq", "state_x", "wq", "wq_t", "state_w"):
                assert same_bits(getattr(bufs, name), getattr(ref_bufs, name)), name
        assert abs(bufs.state_w.item()) > 0


def test_forward_static_empty_batch_and_limits():
    gen = torch.Generator(device=DEV)
    gen.manual_seed(72)
    w = draw(gen, (64, 128), 0.1)
    bufs, ref = sb.LayerBuffers(0, 128, 64, DEV), sb.LayerBuffers(0, 128, 64, DEV)
    x = torch.empty((0, 128), dtype=torch.bfloat16, device=DEV)
    sb.forward(x, w, bufs=ref)
    y, _ = sb.forward_static(x, w, bufs)
    torch.cuda.synchronize()
    assert y.shape == (0, 64)
    for name in ("wq", "wq_t", "state_w"):
        assert same_bits(getattr(bufs, name), getattr(ref, name)), name
    # beyond the stated maximum (2^28 weights) the call refuses before any launch; pointers are never dereferenced
    lib = sb.load_library()
    import ctypes
    fake = ctypes.c_void_p(0x1000)
    saved = sb.SbSaved(0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    assert lib.switchback_forward_static(fake, fake, 8, 16384, 16448, fake, 0, ctypes.byref(saved), None) == 2
    assert lib.switchback_forward_static(fake, fake, 8, 100, 64, fake, 0, ctypes.byref(saved), None) == 2
    assert lib.switchback_forward_static(None, fake, 8, 64, 64, fake, 0, ctypes.byref(saved), None) == 1


def test_a_whole_step_replays_from_a_hip_graph():
    """What the allocation-free forward is for: forward, input gradient and weight gradient of a layer captured into one
    HIP graph (the library only enqueues kernels; it neither allocates, synchronizes nor records memset nodes).  Every
    replay, with eager work and synchronizations in between, must reproduce the eager results bit for bit."""
    gen = torch.Generator(device=DEV)
    gen.manual_seed(73)
    b, n, m = 1500, 1280, 2304
    x, w, dy = draw(gen, (b, n), 1.0), draw(gen, (m, n), 0.03), draw(gen, (b, m), 0.1)
    bufs = sb.LayerBuffers(b, n, m, DEV)
    y, dx, dw = (torch.empty(s, dtype=torch.bfloat16, device=DEV) for s in ((b, m), (b, n), (m, n)))

    def step():
        sb.forward_static(x, w, bufs, y=y)
        sb.backward_input(dy, bufs, dx=dx)
        sb.backward_weight(dy, x, bufs, dw=dw)

    step()                                                        # warm-up: one-time kernel attributes are set here
    torch.cuda.synchronize()
    ref = [t.clone() for t in (y, dx, dw, bufs.xq, bufs.gq, bufs.wq_t, bufs.state_w)]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (y, dx, dw, bufs.xq, bufs.gq, bufs.wq_t):
            t.fill_(1)                                            # eager work between the replays
        bufs.state_w.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for want, got in zip(ref, (y, dx, dw, bufs.xq, bufs.gq, bufs.wq_t, bufs.state_w)):
            assert same_bits(want, got), "replay %d differs from the eager step" % rep
