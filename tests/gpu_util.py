"""Helpers of the GPU tests: torch is used for device memory and streams only."""
import numpy as np
import torch

from paper_2410_09426_amd import binding as fq


def dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor with the same bytes (fp16 goes through a uint16 view)."""
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.uint16).copy()).view(torch.float16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_f16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().view(torch.int16).numpy().view(np.float16)


def run_tq(x, P1, P2, clip, clip_mode, n1, n2, x_stride=None, poison=0xCD, guard=64):
    """Launch the fused kernel on device tensors; returns (codes u8 [T, n/2], scales fp16 [T]) on the host.
    Outputs sit inside poisoned guard bands that must come back untouched."""
    T = x.shape[0]
    n = n1 * n2
    xs = x.stride(0) if x_stride is None else x_stride
    cbuf = torch.full((guard + T * (n // 2) + guard,), poison, dtype=torch.uint8, device="cuda")
    sg = guard + (guard & 1)          # fp16 steps need a 2-byte aligned address
    sbuf = torch.full((sg + T * 2 + sg,), poison, dtype=torch.uint8, device="cuda")
    codes = cbuf[guard:guard + T * (n // 2)]
    scales = sbuf[sg:sg + T * 2]
    fq.flatquant_transform_quant(x, P1, P2, clip, clip_mode, T, n1, n2, xs, codes, scales,
                                 stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for b, g in ((cbuf, guard), (sbuf, sg)):
        assert bool((b[:g] == poison).all()) and bool((b[-g:] == poison).all()), "guard band overwritten"
    return codes.cpu().numpy().reshape(T, n // 2), scales.cpu().numpy().view(np.float16).reshape(T), codes, scales


def run_dequant(codes_dev, scales_dev, zeros_dev, rows, n, bits=None):
    out = torch.full((rows, n), float("nan"), dtype=torch.float32, device="cuda")
    if bits is None:
        fq.flatquant_dequant(codes_dev, scales_dev, zeros_dev, rows, n, out, stream=torch.cuda.current_stream())
    else:
        fq.flatquant_dequant_bits(codes_dev, scales_dev, zeros_dev, rows, n, bits, out, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()
