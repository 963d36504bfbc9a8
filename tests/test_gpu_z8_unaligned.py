"""GPU parity of the entry points for operands the pipelined loops cannot take as they are:
N and K that are not multiples of 8, odd row pitches and batch strides, base addresses aligned to
one element only, convolutions with 3 input channels.  Exact on integers, within the acceptance
bound on random data, and the bytes of C around the valid elements stay as they were."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import ADT, DEV, ODT, TDT, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _embed(t, offset, row_pad, batch_pad=0, fill=0.0):
    """t as a view into a larger 1-D device buffer: base `offset` elements in, rows `row_pad` and
    batch entries `batch_pad` elements longer than their data.  Returns (view, buffer)."""
    rows, cols = t.shape[-2:]
    pitch = cols + row_pad
    per = rows * pitch + batch_pad
    b = t.shape[0] if t.dim() == 3 else 1
    buf = torch.full((offset + b * per,), fill, dtype=t.dtype, device=DEV)
    if t.dim() == 3:
        view = buf[offset:].as_strided((b, rows, cols), (per, pitch, 1))
    else:
        view = buf[offset:].as_strided((rows, cols), (pitch, 1))
    view.copy_(t.to(DEV))
    return view, buf


def _untouched(buf, view):
    mask = torch.ones_like(buf, dtype=torch.bool)
    off = (view.data_ptr() - buf.data_ptr()) // buf.element_size()
    mask[off:].as_strided(view.shape, view.stride()).fill_(False)
    return bool(torch.isnan(buf[mask]).all())


def _ws(nbytes):
    assert nbytes > 0
    return torch.empty(nbytes, dtype=torch.uint8, device=DEV)


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("dt,out", [("f16", "f16"), ("bf16", "f32")])
def test_gemm_integers_bit_exact_odd_everything(dt, out, transA, transB):
    for n, (M, N, K) in enumerate(((37, 29, 45), (301, 203, 515), (1, 1, 1), (129, 7, 1030))):
        A0 = wl.small_ints((K, M) if transA else (M, K), dt, 8100 + n)
        B0 = wl.small_ints((N, K) if transB else (K, N), dt, 8200 + n)
        A, _ = _embed(A0, 1, 3)
        B, _ = _embed(B0, 3, 1)
        C, Cbuf = _embed(torch.zeros(M, N, dtype=TDT[out]), 1, 2, fill=float("nan"))
        C.fill_(float("nan"))
        ws = _ws(al.alcop_unaligned_workspace_bytes(1, M, N, K, ADT[out]))
        al.alcop_bmm_unaligned(A, B, C, ws, transA=bool(transA), transB=bool(transB))
        torch.cuda.synchronize()
        ref = oracle.gemm(wl.bits(A0), wl.bits(B0), ODT[dt], bool(transA), bool(transB))
        assert np.array_equal(to_f64(C), ref), (M, N, K)
        assert _untouched(Cbuf, C), (M, N, K)


def test_batched_random_with_bias_relu_every_kind_of_schedule():
    b, M, N, K = 5, 190, 93, 203
    A0 = wl.uniform((b, M, K), "f16", 8301)
    B0 = wl.uniform((b, K, N), "f16", 8302)
    A, _ = _embed(A0, 1, 1, batch_pad=5)
    B, _ = _embed(B0, 0, 3, batch_pad=1)
    C, Cbuf = _embed(torch.zeros(b, M, N, dtype=torch.float16), 1, 0, batch_pad=3, fill=float("nan"))
    bias0 = torch.linspace(-1.0, 1.0, N)
    bias = torch.full((N + 1,), float("nan"), device=DEV)[1:]
    bias.copy_(bias0.to(DEV))
    ws = _ws(al.alcop_unaligned_workspace_bytes(b, M, N, K, al.F16))
    ref = oracle.epilogue(oracle.bmm(wl.bits(A0), wl.bits(B0), oracle.F16), 0.5, bias0.double().numpy(), 1)
    padded = al.problem(al.OP_BMM, 192, 96, 208, al.F16, al.F16, batch=b)
    space = [s for s in al.alcop_sched_space(padded) if al.alcop_sched_supported(padded, s) == al.OK]
    picks = [None, next(s for s in space if s.variant == 2), next(s for s in space if s.variant == 0 and s.stages == 4)]
    for s in picks:
        C.fill_(float("nan"))
        al.alcop_bmm_unaligned(A, B, C, ws, 0.5, bias, 1, s)
        torch.cuda.synchronize()
        assert_close(to_f64(C), ref, repr(s))
        assert _untouched(Cbuf, C), repr(s)


def test_same_bits_as_the_plain_entry_point_when_the_operands_are_aligned():
    M, N, K = 520, 264, 328
    A = wl.uniform((M, K), "bf16", 8401).to(DEV)
    B = wl.uniform((K, N), "bf16", 8402).to(DEV)
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    C1 = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    C2 = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    ws = _ws(al.alcop_unaligned_workspace_bytes(1, M, N, K, al.BF16))
    al.alcop_gemm(A, B, C1, s)
    al.alcop_bmm_unaligned(A, B, C2, ws, sched=s)
    torch.cuda.synchronize()
    assert torch.equal(C1.view(torch.int16), C2.view(torch.int16))


@pytest.mark.parametrize("C,K,hw,stride,pad,dil", [(3, 64, (57, 49), (2, 2), (3, 3), (1, 1)),   # a 7x7 stem
                                                    (5, 12, (19, 23), (1, 1), (2, 2), (2, 2)),
                                                    (24, 3, (16, 16), (1, 2), (0, 1), (1, 1))])
def test_convolution_any_channel_counts(C, K, hw, stride, pad, dil):
    R = 7 if C == 3 else 3
    x0 = wl.small_ints((4, hw[0], hw[1], C), "f16", 8500 + C)
    w0 = wl.small_ints((R, R, C, K), "f16", 8600 + K)
    ref = oracle.conv2d(wl.bits(x0), wl.bits(w0), oracle.F16, stride, pad, dil)
    bias0 = torch.arange(K, dtype=torch.float32) - 2
    ref = oracle.epilogue(ref.reshape(-1, K), 1.0, bias0.double().numpy(), 0).reshape(ref.shape)
    x = torch.zeros(x0.numel() + 1, dtype=torch.float16, device=DEV)[1:].view(x0.shape)
    x.copy_(x0.to(DEV))
    w = torch.zeros(w0.numel() + 1, dtype=torch.float16, device=DEV)[1:].view(w0.shape)
    w.copy_(w0.to(DEV))
    yb = torch.full((ref.size + 2,), float("nan"), dtype=torch.float32, device=DEV)
    y = yb[1:-1].view(ref.shape)
    bias = bias0.to(DEV)
    ws = _ws(al.alcop_conv2d_unaligned_workspace_bytes(4, hw[0], hw[1], C, K, R, R, stride, pad, dil, al.F32))
    al.alcop_conv2d_igemm_unaligned(x, w, y, ws, stride, pad, dil, 1.0, bias, 0)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(y), ref)
    assert bool(torch.isnan(yb[0])) and bool(torch.isnan(yb[-1]))


def test_refusals_reach_no_kernel():
    A = wl.small_ints((9, 11), "f16", 1).to(DEV)
    B = wl.small_ints((11, 10), "f16", 2).to(DEV)
    C = torch.full((9, 10), float("nan"), dtype=torch.float16, device=DEV)
    need = al.alcop_unaligned_workspace_bytes(1, 9, 10, 11, al.F16)
    with pytest.raises(al.AlcopError) as e:
        al.alcop_bmm_unaligned(A, B, C, _ws(need - 1))
    assert e.value.code == al.ERR_SIZE
    with pytest.raises(al.AlcopError) as e:
        al.alcop_bmm_unaligned(A, B, C, torch.empty(need + 16, dtype=torch.uint8, device=DEV)[1:need + 1])
    assert e.value.code == al.ERR_ALIGN
    torch.cuda.synchronize()
    assert bool(torch.isnan(C).all())
