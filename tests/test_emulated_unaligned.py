"""Entry points for operands the pipelined loops cannot take as they are (N, K not multiples of
8, odd pitches, element-aligned base addresses, a 3-channel image), run on the CPU model of the
hardware: the pack and unpack kernels and the product between them must stay inside the
operands and the workspace, leave the padding of C alone, and equal the oracle exactly."""
import numpy as np
import pytest
import torch

import emu_util as emu
import oracle
import paper_2210_16691_amd as al
import workloads as wl

TDT = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}
ODT = {"f16": oracle.F16, "bf16": oracle.BF16}
ADT = {"f16": al.F16, "bf16": al.BF16, "f32": al.F32}


def _embed(t, offset, row_pad, batch_pad=0, fill=0.0):
    """A copy of t (2-D or 3-D) as a view into a larger 1-D buffer: base address `offset` elements
    into it, rows `row_pad` elements apart beyond their length, batch entries `batch_pad` beyond
    theirs.  Returns (view, buffer)."""
    rows, cols = t.shape[-2:]
    pitch = cols + row_pad
    per = rows * pitch + batch_pad
    b = t.shape[0] if t.dim() == 3 else 1
    buf = torch.full((offset + b * per,), fill, dtype=t.dtype)
    if t.dim() == 3:
        view = buf[offset:].as_strided((b, rows, cols), (per, pitch, 1))
    else:
        view = buf[offset:].as_strided((rows, cols), (pitch, 1))
    view.copy_(t)
    return view, buf


def _workspace(nbytes):
    return torch.empty(nbytes + 16, dtype=torch.uint8)[:nbytes] if nbytes % 16 else torch.empty(nbytes, dtype=torch.uint8)


def _untouched(buf, view):
    """True if every element of buf outside the view is still NaN."""
    mask = torch.ones_like(buf, dtype=torch.bool)
    off = (view.data_ptr() - buf.data_ptr()) // buf.element_size()
    m = mask[off:].as_strided(view.shape, view.stride())
    m.fill_(False)
    return bool(torch.isnan(buf[mask]).all())


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("dt,out", [("f16", "f16"), ("bf16", "f32")])
def test_gemm_odd_extents_pitches_and_addresses(dt, out, transA, transB):
    M, N, K = 37, 29, 45
    A0 = wl.small_ints((K, M) if transA else (M, K), dt, 7100 + transA)
    B0 = wl.small_ints((N, K) if transB else (K, N), dt, 7200 + transB)
    A, _ = _embed(A0, 1, 3)
    B, _ = _embed(B0, 3, 1)
    C, Cbuf = _embed(torch.zeros(M, N, dtype=TDT[out]), 1, 2, fill=float("nan"))
    C.fill_(float("nan"))
    ws = _workspace(al.alcop_unaligned_workspace_bytes(1, M, N, K, ADT[out]))
    ref = oracle.gemm(wl.bits(A0), wl.bits(B0), ODT[dt], bool(transA), bool(transB))
    padded = al.problem(al.OP_GEMM, 40, 32, 48, ADT[dt], ADT[out], transB=bool(transB), transA=bool(transA))
    for sched, policy in ((None, (1, 0)), (emu.space(padded)[-1], (0, 1))):
        C.fill_(float("nan"))
        errs = emu.call(al.alcop_bmm_unaligned, A, B, C, ws, sched=sched, transA=bool(transA),
                        transB=bool(transB), reads=[A, B], writes=[C, ws], policy=policy)
        assert not errs, errs[:4]
        assert np.array_equal(C.double().numpy(), ref)
        assert _untouched(Cbuf, C)


def test_batched_with_bias_relu_and_a_persistent_schedule():
    b, M, N, K = 3, 70, 21, 19
    A0 = wl.small_ints((b, M, K), "f16", 7301)
    B0 = wl.small_ints((b, K, N), "f16", 7302)
    A, _ = _embed(A0, 1, 1, batch_pad=5)
    B, _ = _embed(B0, 0, 3, batch_pad=1)
    C, Cbuf = _embed(torch.zeros(b, M, N, dtype=torch.float16), 1, 0, batch_pad=3, fill=float("nan"))
    C.fill_(float("nan"))
    bias_buf = torch.full((N + 1,), float("nan"), dtype=torch.float32)
    bias = bias_buf[1:]                      # 4-byte aligned only
    bias.copy_(torch.arange(N, dtype=torch.float32) % 5 - 2)
    ws = _workspace(al.alcop_unaligned_workspace_bytes(b, M, N, K, al.F16))
    ref = oracle.epilogue(oracle.bmm(wl.bits(A0), wl.bits(B0), oracle.F16), 0.5, bias.double().numpy(), 1)
    padded = al.problem(al.OP_BMM, 72, 24, 24, al.F16, al.F16, batch=b)
    persistent = [s for s in emu.space(padded) if s.variant == 2]
    assert persistent
    for sched in (None, persistent[0]):
        C.fill_(float("nan"))
        errs = emu.call(al.alcop_bmm_unaligned, A, B, C, ws, 0.5, bias, 1, sched, reads=[A, B, bias],
                        writes=[C, ws], policy=(1, 1))
        assert not errs, errs[:4]
        assert np.array_equal(C.double().numpy(), ref)
        assert _untouched(Cbuf, C)


def test_aligned_operands_give_the_same_bits_as_the_plain_entry_point():
    M, N, K = 72, 64, 96
    A = wl.uniform((M, K), "f16", 7401)
    B = wl.uniform((K, N), "f16", 7402)
    s = al.sched(64, 64, 64, 32, 32, 3, 2, 1)
    C1 = torch.empty(M, N, dtype=torch.float16)
    C2 = torch.empty(M, N, dtype=torch.float16)
    ws = _workspace(al.alcop_unaligned_workspace_bytes(1, M, N, K, al.F16))
    assert not emu.call(al.alcop_gemm, A, B, C1, s, reads=[A, B], writes=[C1])
    assert not emu.call(al.alcop_bmm_unaligned, A, B, C2, ws, sched=s, reads=[A, B], writes=[C2, ws])
    assert torch.equal(C1.view(torch.int16), C2.view(torch.int16))


@pytest.mark.parametrize("C,K,stride,pad,dil", [(3, 5, (2, 2), (1, 1), (1, 1)), (5, 12, (1, 1), (2, 2), (2, 2)),
                                                 (8, 3, (1, 2), (0, 1), (1, 1))])
def test_convolution_any_channel_counts(C, K, stride, pad, dil):
    x0 = wl.small_ints((2, 9, 8, C), "f16", 7500 + C)
    w0 = wl.small_ints((3, 3, C, K), "f16", 7600 + K)
    ref = oracle.conv2d(wl.bits(x0), wl.bits(w0), oracle.F16, stride, pad, dil)
    bias = torch.arange(K, dtype=torch.float32) - 2
    ref = oracle.epilogue(ref.reshape(-1, K), 1.0, bias.double().numpy(), 0).reshape(ref.shape)
    # element-aligned placement: each tensor one element into its buffer
    xb = torch.zeros(x0.numel() + 1, dtype=torch.float16)
    x = xb[1:].view(x0.shape)
    x.copy_(x0)
    wb = torch.zeros(w0.numel() + 1, dtype=torch.float16)
    w = wb[1:].view(w0.shape)
    w.copy_(w0)
    yb = torch.full((ref.size + 2,), float("nan"), dtype=torch.float16)
    y = yb[1:-1].view(ref.shape)
    ws = _workspace(al.alcop_conv2d_unaligned_workspace_bytes(2, 9, 8, C, K, 3, 3, stride, pad, dil, al.F16))
    errs = emu.call(al.alcop_conv2d_igemm_unaligned, x, w, y, ws, stride, pad, dil, 1.0, bias, 0,
                    reads=[x, w, bias], writes=[y, ws], policy=(0, 1))
    assert not errs, errs[:4]
    assert np.array_equal(y.double().numpy(), ref)
    assert torch.isnan(yb[0]) and torch.isnan(yb[-1])


def test_workspace_rules():
    M, N, K = 9, 10, 11
    A = wl.small_ints((M, K), "f16", 1)
    B = wl.small_ints((K, N), "f16", 2)
    C = torch.empty(M, N, dtype=torch.float16)
    need = al.alcop_unaligned_workspace_bytes(1, M, N, K, al.F16)
    # three padded images (16 x 16 halves each, rounded to 256 bytes) and the bias
    assert need == 3 * 512 + 256
    assert al.alcop_unaligned_workspace_bytes(0, M, N, K, al.F16) == 0
    assert al.alcop_unaligned_workspace_bytes(1, M, N, K, 7) == 0
    assert al.alcop_conv2d_unaligned_workspace_bytes(1, 2, 2, 3, 3, 3, 3, (1, 1), (0, 0), (1, 1), al.F16) == 0
    small = torch.empty(need - 1, dtype=torch.uint8)
    with pytest.raises(al.AlcopError) as e:
        emu.call(al.alcop_bmm_unaligned, A, B, C, small, reads=[A, B], writes=[C, small])
    assert e.value.code == al.ERR_SIZE
    odd = torch.empty(need + 16, dtype=torch.uint8)[1:need + 1]
    with pytest.raises(al.AlcopError) as e:
        emu.call(al.alcop_bmm_unaligned, A, B, C, odd, reads=[A, B], writes=[C, odd])
    assert e.value.code == al.ERR_ALIGN
