"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function include/switchback.h
declares, sizes workspaces, and rejects bad arguments before any kernel launch."""
import ctypes
import os
import re

import pytest

from paper_2304_13013_amd import switchback as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sb.LIB_PATH):
        from paper_2304_13013_amd import build
        build.build()
    return sb.load_library()


def declared_functions():
    """Every function any header under include/ declares."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if header.endswith(".h"):
            with open(os.path.join(inc, header)) as fh:
                text = re.sub(r"/\*.*?\*/", "", fh.read(), flags=re.S)
            names |= set(re.findall(r"\b(switchback_\w+)\s*\(", text))
    return sorted(names)


def test_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"switchback_quantize_rowwise", "switchback_quantize_tensorwise", "switchback_forward",
            "switchback_backward_input", "switchback_backward_weight", "switchback_forward_static",
            "switchback_ceiling_mfma", "switchback_ceiling_copy"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = {lib.switchback_status_string(i).decode() for i in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert "unknown" in lib.switchback_status_string(99).decode()


def test_workspace_sizes(lib):
    assert sb.workspace_bytes(sb.SB_OP_FORWARD, 512, 256, 1024) >= 4096
    assert sb.workspace_bytes(sb.SB_OP_QUANTIZE_TENSORWISE, 0, 256, 1024) >= 4096
    assert sb.workspace_bytes(sb.SB_OP_BACKWARD_INPUT, 512, 256, 1024) == 0
    big = sb.workspace_bytes(sb.SB_OP_BACKWARD_WEIGHT, 32896, 1280, 1280)
    assert big % (1280 * 1280 * 4) == 0          # whole binary32 partial matrices
    assert sb.workspace_bytes(sb.SB_OP_BACKWARD_WEIGHT, 16384, 4096, 16384) == 0  # enough tiles, no split
    assert sb.workspace_bytes(sb.SB_OP_QUANTIZE_COLWISE, 0, 1280, 5120) == 64 * 1280 * 2   # 64 row runs of 16-bit maxima
    assert sb.workspace_bytes(sb.SB_OP_QUANTIZE_COLWISE, 0, 64, 32) == 2 * 64 * 2
    assert sb.workspace_bytes(sb.SB_OP_STABLE_ADAMW, 0, 0, 0) == 2048 * 8                  # binary64 partial sums
    assert sb.workspace_bytes(99, 1, 64, 64) == 0


def test_bad_arguments_are_rejected_before_launch(lib):
    """Every call below must return an error code without touching the GPU (there is none on the build box)."""
    fake = ctypes.c_void_p(0x1000)               # aligned, never dereferenced on the host
    odd = ctypes.c_void_p(0x1004)
    null = ctypes.c_void_p(None)
    saved = sb.SbSaved(0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    sp = ctypes.byref(saved)
    INVALID, SHAPE, WS = 1, 2, 3
    assert lib.switchback_quantize_rowwise(null, 4, 64, fake, fake, null) == INVALID
    assert lib.switchback_quantize_rowwise(odd, 4, 64, fake, fake, null) == INVALID
    assert lib.switchback_quantize_rowwise(fake, -1, 64, fake, fake, null) == INVALID
    assert lib.switchback_quantize_rowwise(fake, 4, 60, fake, fake, null) == SHAPE
    assert lib.switchback_quantize_rowwise(fake, 4, 1 << 20, fake, fake, null) == SHAPE
    assert lib.switchback_quantize_rowwise(null, 0, 64, null, null, null) == 0       # empty input: no-op
    assert lib.switchback_quantize_tensorwise(fake, 64, 64, fake, fake, fake, fake, 16, null) == WS
    assert lib.switchback_quantize_tensorwise(fake, 64, 72, fake, fake, fake, fake, 1 << 20, null) == SHAPE
    assert lib.switchback_quantize_tensorwise(fake, 64, 64, fake, odd, fake, fake, 1 << 20, null) == INVALID
    assert lib.switchback_matmul_int8_dequant(fake, fake, fake, fake, 8, 64, 32, fake, 0, null) == SHAPE
    assert lib.switchback_matmul_int8_dequant(fake, fake, fake, fake, 8, 64, 1 << 18, fake, 0, null) == SHAPE
    assert lib.switchback_matmul_int8_dequant(fake, null, fake, fake, 8, 64, 64, fake, 0, null) == INVALID
    assert lib.switchback_matmul_int8_dequant(fake, fake, fake, fake, 8, 64, 64, fake, 7, null) == INVALID
    assert lib.switchback_forward(fake, fake, 8, 100, 64, fake, 0, sp, fake, 1 << 20, null) == SHAPE
    assert lib.switchback_forward(fake, fake, 8, 64, 64, fake, 0, None, fake, 1 << 20, null) == INVALID
    assert lib.switchback_forward(fake, fake, 8, 64, 64, fake, 0, sp, fake, 8, null) == WS
    assert lib.switchback_forward(null, fake, 8, 64, 64, fake, 0, sp, fake, 1 << 20, null) == INVALID
    assert lib.switchback_backward_input(fake, sp, 8, 64, 96, fake, 0, fake, fake, null) == SHAPE
    assert lib.switchback_backward_input(null, sp, 8, 64, 64, fake, 0, fake, fake, null) == INVALID
    assert lib.switchback_backward_input(null, sp, 0, 64, 64, null, 0, null, null, null) == 0   # b = 0
    assert lib.switchback_quantize_colwise_transpose(fake, 64, 64, fake, fake, fake, 16, null) == WS
    assert lib.switchback_quantize_colwise_transpose(fake, 64, 72, fake, fake, fake, 1 << 20, null) == SHAPE
    assert lib.switchback_quantize_colwise_transpose(fake, 64, 64, odd, fake, fake, 1 << 20, null) == INVALID
    assert lib.switchback_matmul_int8_dequant_rc(fake, fake, fake, fake, 8, 64, 32, fake, 0, null) == SHAPE
    assert lib.switchback_matmul_int8_dequant_rc(fake, fake, fake, null, 8, 64, 64, fake, 0, null) == INVALID
    assert lib.switchback_matmul_int8_dequant_rc(fake, fake, fake, fake, 8, 64, 64, fake, 2, null) == INVALID
    assert lib.switchback_forward_q(fake, fake, 8, 100, 64, fake, 0, fake, fake, fake, fake, null) == SHAPE
    assert lib.switchback_forward_q(fake, fake, 8, 64, 64, fake, 0, fake, fake, null, fake, null) == INVALID
    assert lib.switchback_backward_input_q(fake, fake, 8, 64, 64, fake, 0, fake, fake, fake, fake, fake, 8, null) == WS
    assert lib.switchback_backward_input_q(fake, null, 8, 64, 64, fake, 0, fake, fake, fake, fake, fake, 1 << 20, null) == INVALID
    assert lib.switchback_dequantize_rowwise(fake, fake, 4, 60, fake, null) == SHAPE
    assert lib.switchback_dequantize_rowwise(fake, null, 4, 64, fake, null) == INVALID
    assert lib.switchback_dequantize_rowwise(null, null, 0, 64, null, null) == 0          # empty input: no-op
    assert lib.switchback_backward_weight_m(fake, sp, 8, 64, 64, null, fake, 0, fake, 1 << 30, null) == INVALID
    assert lib.switchback_backward_weight_m(fake, sp, 32896, 1280, 1280, fake, fake, 0, fake, 64, null) == WS
    assert lib.switchback_backward_weight(fake, fake, 8, 64, 64, fake, 2, fake, 1 << 30, null) == INVALID
    assert lib.switchback_backward_weight(fake, fake, 32896, 1280, 1280, fake, 0, fake, 64, null) == WS
    assert lib.switchback_backward_weight(fake, fake, 8, 64, 64, null, 0, fake, 1 << 30, null) == INVALID
    assert lib.switchback_quantize_rowwise_f8(fake, 4, 64, 2, fake, fake, null) == INVALID       # unknown format
    assert lib.switchback_quantize_rowwise_f8(fake, 4, 60, 0, fake, fake, null) == SHAPE
    assert lib.switchback_quantize_rowwise_f8(null, 0, 64, 1, null, null, null) == 0
    assert lib.switchback_quantize_tensorwise_f8(fake, 64, 64, 0, fake, fake, fake, fake, 16, null) == WS
    assert lib.switchback_quantize_tensorwise_f8(fake, 64, 64, 5, fake, fake, fake, fake, 1 << 20, null) == INVALID
    assert lib.switchback_matmul_f8_dequant(fake, 0, fake, fake, 0, fake, 8, 64, 64, fake, 0, null) == SHAPE   # K % 128
    assert lib.switchback_matmul_f8_dequant(fake, 0, fake, fake, 0, fake, 8, 64, 128, fake, 2, null) == INVALID
    assert lib.switchback_matmul_f8_dequant(fake, 0, null, fake, 0, fake, 8, 64, 128, fake, 0, null) == INVALID
    assert lib.switchback_forward_f8(fake, fake, 8, 64, 128, fake, 0, sp, 0, 0, fake, 1 << 20, null) == SHAPE
    assert lib.switchback_forward_f8(fake, fake, 8, 128, 128, fake, 0, sp, 0, 3, fake, 1 << 20, null) == INVALID
    assert lib.switchback_forward_f8(fake, fake, 8, 128, 128, fake, 0, sp, 0, 0, fake, 8, null) == WS
    assert lib.switchback_backward_input_f8(fake, sp, 8, 128, 192, fake, 0, fake, fake, 1, 0, null) == SHAPE
    assert lib.switchback_backward_input_f8(null, sp, 8, 128, 128, fake, 0, fake, fake, 1, 0, null) == INVALID
    assert lib.switchback_backward_input_f8(null, sp, 0, 128, 128, null, 0, null, null, 1, 0, null) == 0
    adam = lib.switchback_stable_adamw_step
    good = (1e-3, 0.9, 0.98, 1e-6, 0.2)
    assert adam(fake, fake, fake, fake, 0, 100, *good, 0, null, fake, 1 << 20, null) == INVALID    # t starts at 1
    assert adam(fake, fake, fake, fake, 2, 100, *good, 1, null, fake, 1 << 20, null) == INVALID    # grad dtype
    assert adam(fake, fake, fake, fake, 0, 100, 1e-3, 1.0, 0.98, 1e-6, 0.2, 1, null, fake, 1 << 20, null) == INVALID
    assert adam(fake, fake, fake, fake, 0, 100, 1e-3, 0.9, 0.98, 0.0, 0.2, 1, null, fake, 1 << 20, null) == INVALID
    assert adam(fake, odd, fake, fake, 0, 100, *good, 1, null, fake, 1 << 20, null) == INVALID
    assert adam(fake, fake, fake, fake, 0, 100, *good, 1, null, fake, 8, null) == WS
    assert adam(null, null, null, null, 0, 0, *good, 1, null, null, 0, null) == 0                  # empty tensor
    table = (sb.SbAdamwTensor * 3)(sb.SbAdamwTensor(0x1000, 0x2000, 0x3000, 0x4000, 5, 0, 0),
                                   sb.SbAdamwTensor(0x1000, 0x2000, 0x3000, 0x4000, 1280 * 5120, 0, 0),
                                   sb.SbAdamwTensor(0x1000, 0x2000, 0x3000, 0x4000, 100 * 1000 * 1000, 0, 0))
    total = lib.switchback_stable_adamw_plan(table, 3)
    assert [t.num_blocks for t in table] == [1, 1600, 2048] and [t.first_block for t in table] == [0, 1, 1601]
    assert total == 3649
    table[1].count = 0
    assert lib.switchback_stable_adamw_plan(table, 3) == -INVALID
    assert lib.switchback_stable_adamw_plan(None, 0) == 0
    multi = lib.switchback_stable_adamw_step_multi
    assert multi(fake, 3, 3649, 0, *good, 1, null, fake, 8 * 3649 - 1, null) == WS
    assert multi(fake, 3, 2, 0, *good, 1, null, fake, 1 << 20, null) == INVALID                    # fewer blocks than tensors
    assert multi(null, 3, 3649, 0, *good, 1, null, fake, 1 << 20, null) == INVALID
    assert multi(fake, 3, 3649, 0, *good, 0, null, fake, 1 << 20, null) == INVALID
    assert multi(null, 0, 0, 0, *good, 1, null, null, 0, null) == 0
    # the allocation-free forward: shape limits first, then pointers; nothing is launched
    assert lib.switchback_forward_static(fake, fake, 8, 16384, 16448, fake, 0, sp, null) == SHAPE   # m * n > 2^28
    assert lib.switchback_forward_static(fake, fake, 8, 100, 64, fake, 0, sp, null) == SHAPE
    assert lib.switchback_forward_static(null, fake, 8, 64, 64, fake, 0, sp, null) == INVALID
    assert lib.switchback_forward_static(fake, fake, 8, 64, 64, fake, 9, sp, null) == INVALID
    bl = lib.switchback_matmul_int8_dequant_bias_layerscale
    assert bl(fake, fake, fake, fake, fake, fake, 8, 64, 32, fake, 0, null) == SHAPE
    assert bl(fake, fake, fake, fake, odd, fake, 8, 64, 64, fake, 0, null) == INVALID               # misaligned bias
    assert bl(fake, fake, fake, fake, null, null, 8, 64, 64, fake, 2, null) == INVALID              # no raw mode
    assert bl(fake, null, fake, fake, null, null, 8, 64, 64, fake, 0, null) == INVALID
    assert bl(null, null, null, null, null, null, 0, 64, 64, null, 0, null) == 0
    fbl = lib.switchback_forward_bias_layerscale
    assert fbl(fake, fake, fake, fake, 8, 100, 64, fake, 0, sp, fake, 1 << 20, null) == SHAPE
    assert fbl(fake, fake, fake, odd, 8, 64, 64, fake, 0, sp, fake, 1 << 20, null) == INVALID
    assert fbl(fake, fake, null, null, 8, 64, 64, fake, 0, sp, fake, 8, null) == WS
    assert fbl(fake, fake, null, null, 8, 64, 64, fake, 2, sp, fake, 1 << 20, null) == INVALID
    # the measurement aids validate their arguments too
    ceil = lib.switchback_ceiling_mfma
    assert ceil(0, fake, 1024, fake, 1024, 0, 8, 10, fake, None, null) == INVALID                   # no workgroups
    assert ceil(0, fake, 1000, fake, 1024, 8, 8, 10, fake, None, null) == INVALID                   # not whole fragments
    assert ceil(2, fake, 1024, fake, 2048, 8, 8, 10, fake, None, null) == INVALID                   # float8 fragments are 2 KiB
    assert ceil(3, fake, 1024, fake, 1024, 8, 8, 10, fake, None, null) == INVALID
    assert ceil(0, fake, 1024, fake, 1024, 8, 5, 10, fake, None, null) == INVALID
    assert lib.switchback_ceiling_copy(fake, odd, 64, null) == INVALID
    assert lib.switchback_ceiling_copy(fake, fake, 24, null) == INVALID
    assert lib.switchback_ceiling_copy(fake, fake, 0, null) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(sb.SwitchBackError):
        sb.quantize_rowwise(torch.zeros(4, 64, dtype=torch.bfloat16))


def test_binding_refuses_buffers_of_another_shape(lib):
    """Caller-supplied layer buffers and outputs must have exactly the shape the kernels will write: the binding raises
    before any launch (CPU tensors here, so a call that got past the check would raise on the device test instead, with a
    different message)."""
    import torch
    z = lambda *shape, dt=torch.bfloat16: torch.zeros(shape, dtype=dt)
    bufs = sb.LayerBuffers(8, 64, 128, "cpu")
    for call in (lambda: sb.forward(z(16, 64), z(128, 64), bufs=bufs),                   # b differs
                 lambda: sb.forward(z(8, 64), z(192, 64), bufs=bufs),                    # m differs
                 lambda: sb.backward_input(z(8, 192), bufs),                             # m differs
                 lambda: sb.backward_weight(z(16, 128), z(16, 64), bufs),                # b differs
                 lambda: sb.backward_weight_m(z(8, 64), bufs),                           # m differs
                 lambda: sb.forward_f8(z(8, 128), z(128, 128), bufs=bufs),               # n differs
                 lambda: sb.backward_input_f8(z(4, 128), bufs)):                         # b differs
        with pytest.raises(sb.SwitchBackError, match="allocated for"):
            call()
    qbufs = sb.LayerBuffersQ(8, 64, 128, "cpu")
    with pytest.raises(sb.SwitchBackError, match="allocated for"):
        sb.forward_q(z(8, 64), z(64, 64), bufs=qbufs)
    with pytest.raises(sb.SwitchBackError, match="allocated for"):
        sb.backward_input_q(z(9, 128), z(128, 64), qbufs)
    for call in (lambda: sb.forward(z(8, 64), z(128, 64), bufs=bufs, y=z(8, 64)),        # y too narrow
                 lambda: sb.forward(z(8, 64), z(128, 64), bufs=bufs, y=z(8, 128, dt=torch.float32)),   # dtype
                 lambda: sb.backward_input(z(8, 128), bufs, dx=z(4, 64)),
                 lambda: sb.backward_weight(z(8, 128), z(8, 64), bufs, dw=z(64, 128)),   # transposed
                 lambda: sb.backward_weight_m(z(8, 128), bufs, x_hat=z(8, 32)),
                 lambda: sb.quantize_rowwise(z(8, 64), q=z(8, 32, dt=torch.int8)),
                 lambda: sb.quantize_rowwise(z(8, 64), state=z(4, dt=torch.float32)),
                 lambda: sb.quantize_tensorwise(z(64, 32), q_t=z(64, 32, dt=torch.int8)),
                 lambda: sb.dequantize_rowwise(z(8, 64, dt=torch.int8), z(8, dt=torch.float32), out=z(8, 32)),
                 lambda: sb.quantize_colwise_transpose(z(64, 32), q_t=z(64, 32, dt=torch.int8)),
                 lambda: sb.matmul_int8_dequant(z(8, 64, dt=torch.int8), z(8, dt=torch.float32),
                                                z(64, 64, dt=torch.int8), z(1, dt=torch.float32), out=z(8, 32)),
                 lambda: sb.matmul_int8_dequant(z(8, 64, dt=torch.int8), z(4, dt=torch.float32),
                                                z(64, 64, dt=torch.int8), z(1, dt=torch.float32)),
                 lambda: sb.matmul_int8_dequant_rc(z(8, 64, dt=torch.int8), z(8, dt=torch.float32),
                                                   z(64, 64, dt=torch.int8), z(32, dt=torch.float32)),
                 lambda: sb.matmul_f8_dequant(z(8, 128, dt=torch.uint8), 0, z(8, dt=torch.float32),
                                              z(64, 128, dt=torch.uint8), 0, z(1, dt=torch.float32), out=z(8, 32))):
        with pytest.raises(sb.SwitchBackError, match="must be a"):
            call()


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch):
    """The product path has no CPU fallback: without the built library every entry point of the binding raises."""
    monkeypatch.setattr(sb, "_lib", None)
    monkeypatch.setattr(sb, "LIB_PATH", os.path.join(ROOT, "paper_2304_13013_amd", "no_such_library.so"))
    with pytest.raises(sb.SwitchBackError):
        sb.load_library()
    with pytest.raises(sb.SwitchBackError):
        sb.workspace_bytes(sb.SB_OP_FORWARD, 8, 64, 64)
