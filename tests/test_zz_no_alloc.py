"""civic_decode_attn_noalloc (the entry point for callers that cannot allocate) against civic_decode_attn, through
the C ABI: same kernels, so the outputs must agree bit for bit; two calls in a row, the second with a smaller input
(the library's static scratch keeps the first call's contents); sizes beyond the static maximum are rejected."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2605_28115_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bd():
    from paper_2605_28115_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def raw_noalloc(bd, q, kc, vc, n_ctx, out):
    """The raw C symbol: pointers and sizes only."""
    b, hq, d = q.shape
    return bd.lib.civic_decode_attn_noalloc(C.c_void_p(q.data_ptr()), C.c_void_p(kc.data_ptr()), C.c_void_p(vc.data_ptr()),
                                            C.c_void_p(out.data_ptr()), bd.CIVIC_BF16 if q.dtype == torch.bfloat16 else bd.CIVIC_F32,
                                            b, hq, kc.shape[1], d, kc.shape[2], n_ctx, C.c_float(0.0),
                                            C.c_void_p(torch.cuda.current_stream().cuda_stream))


def test_noalloc_equals_the_workspace_call_twice_in_a_row(bd):
    gen = torch.Generator(device="cuda").manual_seed(5)
    cases = [((4, 32, 8, 128), 938, torch.bfloat16),      # 15 splits of the context: the scratch is used
             ((2, 8, 2, 128), 300, torch.bfloat16),       # smaller, right after: stale partial results lie behind its own
             ((1, 4, 2, 64), 50, torch.float32),          # one split: no scratch at all
             ((3, 16, 4, 64), 2000, torch.float32)]
    outs = []
    for (b, hq, hkv, d), n, dt in cases:
        q = torch.randn((b, hq, d), device="cuda", generator=gen).to(dt)
        kc = torch.randn((b, hkv, n + 5, d), device="cuda", generator=gen).to(dt)
        vc = torch.randn((b, hkv, n + 5, d), device="cuda", generator=gen).to(dt)
        out = torch.empty_like(q)
        ref = bd.civic_decode_attn(q, kc, vc, n)                  # (also loads the library's code object on first use)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        assert raw_noalloc(bd, q, kc, vc, n, out) == bd.CIVIC_OK
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before        # the call took no device memory
        assert torch.equal(out, ref), ((b, hq, hkv, d), n, dt)
        outs.append((q, kc, vc, n, out))
    # and against the oracle, so that the pair cannot be wrong together
    q, kc, vc, n, out = outs[1]
    w32 = lambda t: t.float().cpu().numpy()
    ref = oracle.decode_attention(w32(q), w32(kc), w32(vc), n)
    assert np.abs(w32(out).astype(np.float64) - ref).max() <= 2e-2 * max(1.0, float(np.abs(ref).max()))


def test_noalloc_rejects_what_the_static_scratch_cannot_hold(bd):
    b, hq, hkv, d, n = 64, 64, 8, 128, 4096
    need = bd.civic_decode_attn_workspace_bytes(torch.bfloat16, b, hq, hkv, d, n)
    assert need > bd.DECODE_NOALLOC_MAX_BYTES
    fake = C.c_void_p(0x1000)
    rc = bd.lib.civic_decode_attn_noalloc(fake, fake, fake, fake, bd.CIVIC_BF16, b, hq, hkv, d, n, n, C.c_float(0.0), None)
    assert rc == bd.ERR_WORKSPACE
    assert bd.lib.civic_decode_attn_noalloc(None, fake, fake, fake, bd.CIVIC_BF16, 1, 4, 2, 64, 100, 50, C.c_float(0.0), None) == bd.ERR_INVALID_ARG
