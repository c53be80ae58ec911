"""Helpers for the GPU parity tests: device buffers via torch, oracle references."""
import numpy as np
import torch

import oracle
import ntp_inputs as gen
import paper_2412_20379_amd as ntp
from helpers import assert_close, TOL_F32, TOL_BF16

DEV = "cuda:0"


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def dev_bf16_bits(a_f32):
    """float32 array -> device int16 tensor holding its bf16 bit patterns, and the
    float32 values those patterns denote (what both sides aggregate)."""
    bits = gen.to_bf16_bits(a_f32)
    return torch.from_numpy(bits.view(np.int16)).to(DEV), gen.bf16_bits_to_f32(bits)


def host_bf16(t):
    """device int16 tensor of bf16 bit patterns -> float32 numpy values"""
    return gen.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16))


def run_agg(g, x_np, direction="fwd", dtype="f32", chunked=False, ld_in=None, ld_out=None,
            streams=None):
    """Aggregate x_np [n, f] through the library; returns the float32 result [n, f]."""
    n, f = x_np.shape
    ld_in = ld_in or f
    ld_out = ld_out or f
    if dtype == "f32":
        xin = torch.full((n, ld_in), 7.5, dtype=torch.float32, device=DEV)
        xin[:, :f] = dev_f32(x_np)
        out = torch.full((n, ld_out), -3.25, dtype=torch.float32, device=DEV)
        code = ntp.NTP_F32
    else:
        bits, _ = dev_bf16_bits(x_np)
        xin = torch.full((n, ld_in), 0x40F0, dtype=torch.int16, device=DEV)
        xin[:, :f] = bits
        out = torch.full((n, ld_out), 0x4150, dtype=torch.int16, device=DEV)
        code = ntp.NTP_BF16
    torch.cuda.synchronize()
    if chunked:
        cs, xs = streams if streams else (torch.cuda.Stream(), torch.cuda.Stream())
        ntp.ntp_chunked_aggregate(g, ntp.NTP_FWD if direction == "fwd" else ntp.NTP_BWD, xin, out, f, ld_in, ld_out,
                                  code, cs, xs)
    elif direction == "fwd":
        ntp.ntp_aggregate_fwd(g, xin, out, f, ld_in, ld_out, code)
    else:
        ntp.ntp_aggregate_bwd(g, xin, out, f, ld_in, ld_out, code)
    torch.cuda.synchronize()
    if ld_out > f:       # columns outside the slice must be untouched
        pad = out[:, f:].cpu().numpy()
        want = -3.25 if dtype == "f32" else 0x4150
        assert np.all(pad == want), "output columns outside the slice were written"
    res = out[:, :f].contiguous()
    return res.cpu().numpy() if dtype == "f32" else host_bf16(res)


def check_agg(g, og, x_np, direction="fwd", dtype="f32", what="", **kw):
    x_used = x_np if dtype == "f32" else gen.bf16_bits_to_f32(gen.to_bf16_bits(x_np))
    m = og.csr if direction == "fwd" else og.csc
    ref, ref_abs = oracle.aggregate(m, x_used, with_abs=True)
    got = run_agg(g, x_np, direction, dtype, **kw)
    if dtype == "bf16":
        ref = oracle.round_bf16(ref).astype(np.float64)
    assert_close(got, ref, ref_abs, TOL_F32 if dtype == "f32" else TOL_BF16, what)
    return got
