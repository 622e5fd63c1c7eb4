"""The norm entry point that allocates nothing (pt_chunk_grad_sqnorm_noalloc) against the existing
entry point (pt_chunk_grad_sqnorm with a context) and against the oracle.

Both run the same kernels in the same fixed order, so sum of squares, norm and non-finite flag must
agree bit for bit; against the oracle's index-order fp64 sum the bar is the norm's (1e-5 relative
asked, 1e-12 asserted).  Two calls in a row share the library's one scratch array: the second, smaller
call must not see anything the first one left behind (partials, per-chunk sums, a raised flag).
"""
import struct

import numpy as np
import pytest
import torch

import oracle as O
from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import synth
from gpu_harness import to_u16

pytestmark = pytest.mark.gpu


def bits(x: float) -> bytes:
    return struct.pack("<d", x)


def make_grads(dtype, C, S, sigma, step, inf_at=None):
    g = torch.zeros(C, S, dtype=dtype, device="cuda")
    n_real = C * S - 24                      # a short zero tail, as the padding of a last chunk
    synth.normal_16(synth.SEED_GRADS, step, 0, 0, n_real, 1e-3, dtype, "cuda", scale=sigma, out=g.view(-1)[:n_real])
    if inf_at is not None:
        g.view(-1).view(torch.int16)[inf_at] = 0x7C00 if dtype == torch.float16 else 0x7F80
    torch.cuda.synchronize()
    return g


def with_context(g, dtype, C, S, sigma):
    """the existing entry point: recompute from the chunks and finalize"""
    pt_dt = B.PT_BF16 if dtype == torch.bfloat16 else B.PT_FP16
    scaler = B.pt_scaler_cfg(sigma, 2.0, 0.5, 2000, 0) if sigma != 1.0 else None
    ctx = B.pt_ctx_create(pt_dt, S, C, scaler)
    try:
        B.pt_chunk_grad_sqnorm(ctx, [g[c] for c in range(C)], 0, C, True)
        rep = B.pt_step_report_read(ctx)
        return rep.sqnorm, rep.norm, rep.found_inf
    finally:
        B.pt_ctx_destroy(ctx)


def without_allocation(g, dtype, C, S, sigma, out, flag):
    pt_dt = B.PT_BF16 if dtype == torch.bfloat16 else B.PT_FP16
    B.pt_chunk_grad_sqnorm_noalloc(g, pt_dt, S, C, sigma, out, flag)


CASES = [
    # (dtype, first call (C, S, inf?), second, smaller call (C, S, inf?), loss scale)
    (torch.bfloat16, (5, 3 * 32768 + 40, False), (2, 32768 + 8, False), 1.0),
    (torch.bfloat16, (3, 1 << 18, True), (3, 4096, False), 1.0),          # a raised flag must not survive
    (torch.float16, (4, 5 * 32768, False), (1, 24 + 8, False), 65536.0),
    (torch.float16, (2, 1 << 16, False), (2, 1 << 15, True), 1024.0),
]


@pytest.mark.parametrize("dtype,first,second,sigma", CASES)
def test_no_alloc_norm_matches_context_norm_two_calls_in_a_row(dtype, first, second, sigma):
    odt = O.BF16 if dtype == torch.bfloat16 else O.FP16
    inputs = []
    for k, (C, S, inf) in enumerate((first, second)):
        inputs.append((C, S, make_grads(dtype, C, S, sigma, step=11 + k, inf_at=(C * S) // 3 if inf else None)))
    # outputs exist before the calls; the entry point itself allocates nothing
    outs = [torch.full((2,), float("nan"), dtype=torch.float64, device="cuda") for _ in inputs]
    flags = [torch.full((1,), -1, dtype=torch.int32, device="cuda") for _ in inputs]
    # set-up call (looks up the scratch array's address, loads the kernels): outside what is measured
    without_allocation(inputs[1][2], dtype, inputs[1][0], inputs[1][1], sigma, outs[1], flags[1])
    outs[1].fill_(float("nan")); flags[1].fill_(-1)
    torch.cuda.synchronize()
    print(f"[no-alloc] {dtype} first {first} second {second} scale {sigma}", flush=True)
    free_before = torch.cuda.mem_get_info()[0]
    for (C, S, g), out, flag in zip(inputs, outs, flags):      # the two calls, back to back on one stream
        without_allocation(g, dtype, C, S, sigma, out, flag)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated by the calls"
    for (C, S, g), out, flag in zip(inputs, outs, flags):
        got_sq, got_norm = (float(x) for x in out.cpu().numpy())
        got_inf = int(flag.cpu().numpy()[0])
        want_sq, want_norm, want_inf = with_context(g, dtype, C, S, sigma)
        assert got_inf == want_inf
        assert bits(got_sq) == bits(want_sq) and bits(got_norm) == bits(want_norm), (got_sq, want_sq)
        words = to_u16(g).reshape(-1)
        assert got_inf == int(O.found_nonfinite(words, odt))
        if not got_inf:
            osq = O.sqnorm(words, odt, loss_scale=sigma, block=S, threads=4)
            assert abs(got_sq - osq) <= 1e-12 * osq
            assert abs(got_norm - np.sqrt(osq)) <= 1e-12 * np.sqrt(osq)


def test_no_alloc_norm_rejects_what_it_cannot_hold():
    g = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.PtError) as e:          # 2^20 blocks of 32768 elements: twice the scratch
        B.pt_chunk_grad_sqnorm_noalloc(g, B.PT_BF16, 1 << 26, 512, 1.0, out, flag)
    assert e.value.status == B.PT_ERR_UNSUPPORTED
    with pytest.raises(B.PtError) as e:
        B.pt_chunk_grad_sqnorm_noalloc(g, B.PT_BF16, 8, 4097, 1.0, out, flag)
    assert e.value.status == B.PT_ERR_UNSUPPORTED
    with pytest.raises(B.PtError) as e:
        B.pt_chunk_grad_sqnorm_noalloc(g, B.PT_BF16, 12, 1, 1.0, out, flag)
    assert e.value.status == B.PT_ERR_ALIGNMENT
    with pytest.raises(B.PtError) as e:
        B.pt_chunk_grad_sqnorm_noalloc(None, B.PT_BF16, 8, 1, 1.0, out, flag)
    assert e.value.status == B.PT_ERR_INVALID_ARG
