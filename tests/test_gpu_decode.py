"""GPU parity of the decode-step attention (civic_decode_attn) against the CPU oracle, through the C ABI.
Bars: bf16 max|out - ref| <= 2e-2 * max(1, max|ref|) (the output is rounded to bf16, 2^-9 relative; logits and sums
are fp32), fp32 <= 1e-4 * max(1, max|ref|)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28115_amd import workloads as wl
from test_gpu_parity import attn_tol, log, to_dev, to_host, widen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bd():
    from paper_2605_28115_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def check_decode(bd, q, kc, vc, n_ctx, dtype, scale=0.0):
    out = to_host(bd.civic_decode_attn(to_dev(q), to_dev(kc), to_dev(vc), n_ctx, scale))
    ref = oracle.decode_attention(widen(q), widen(kc), widen(vc), n_ctx, scale=None if scale == 0.0 else scale)
    got = widen(out).astype(np.float64)
    err = float(np.abs(got - ref).max())
    log("   max abs err", err, "tol", attn_tol(ref, dtype))
    assert np.isfinite(got).all() and err <= attn_tol(ref, dtype)


@pytest.mark.parametrize("name", ["tiny", "2b", "8b", "video"])
def test_decode_matches_oracle_on_workload_caches(bd, name):
    """The cache is the one the prefill of the workload writes (civic_kv_write on the workload's K and V, S_c rows);
    the query is the next token's: every batch item and head, five seeds."""
    w = wl.WORKLOADS[name]
    for trial in range(5):
        log("decode", name, trial)
        (q, _), (k, _), (v, _) = wl.qkv(w, trial)
        s_c = k.shape[1]
        s_max = s_c + 16
        fill = 0x7FC0 if k.dtype == np.uint16 else np.nan          # NaN in the rows beyond the context
        kc = np.full((w.batch, w.n_kv_heads, s_max, w.head_dim), fill, dtype=k.dtype)
        vc = kc.copy()
        dk, dv = to_dev(kc), to_dev(vc)
        bd.civic_kv_write(to_dev(k), to_dev(v), dk, dv, 0)
        qd = np.ascontiguousarray(q[:, -1])                          # [batch, H_q, d]
        out = to_host(bd.civic_decode_attn(to_dev(qd), dk, dv, s_c))
        ref = oracle.decode_attention(widen(qd), widen(to_host(dk)), widen(to_host(dv)), s_c)
        got = widen(out).astype(np.float64)
        err = float(np.abs(got - ref).max())
        log("   max abs err", err)
        assert np.isfinite(got).all() and err <= attn_tol(ref, w.dtype)
        # and it is the last row of the causal prefill over the same K and V
        full = oracle.attention(widen(q), widen(k), widen(v), True, row_step=s_c - 1 if s_c > 1 else 1)
        assert np.abs(got - full[:, s_c - 1]).max() <= attn_tol(ref, w.dtype)


@pytest.mark.parametrize("shape", [
    # batch, H_q, H_kv, d, s_max, n_ctx
    (1, 4, 4, 128, 8, 1), (2, 8, 2, 128, 40, 33), (1, 32, 8, 128, 1000, 938), (3, 6, 2, 64, 300, 257), (1, 16, 16, 72, 1400, 1365),
    (2, 12, 4, 96, 129, 129), (1, 8, 1, 128, 5000, 4097), (1, 2, 2, 256, 700, 513), (2, 3, 1, 32, 64, 64), (1, 64, 4, 128, 600, 511),
    (70, 8, 8, 128, 200, 150), (1, 4, 2, 512, 90, 77),
])
def test_decode_shapes_tails_and_head_dims(bd, shape):
    b, hq, hkv, d, s_max, n = shape
    log("decode shape", shape)
    rng = np.random.default_rng(d + n)
    q = wl.quantize(rng.standard_normal((b, hq, d)).astype(np.float32) * 1.5, "bf16")[0]
    kc = wl.quantize(rng.standard_normal((b, hkv, s_max, d)).astype(np.float32), "bf16")[0]
    vc = wl.quantize(rng.standard_normal((b, hkv, s_max, d)).astype(np.float32), "bf16")[0]
    kc[:, :, n:] = 0x7FC0
    vc[:, :, n:] = 0x7FC0
    check_decode(bd, q, kc, vc, n, "bf16")
    if d <= 128:
        q32 = rng.standard_normal((b, hq, d)).astype(np.float32)
        k32 = rng.standard_normal((b, hkv, s_max, d)).astype(np.float32)
        v32 = rng.standard_normal((b, hkv, s_max, d)).astype(np.float32)
        k32[:, :, n:] = np.nan
        v32[:, :, n:] = np.nan
        check_decode(bd, q32, k32, v32, n, "fp32", scale=0.2)


def test_decode_one_key_per_query_and_large_logits(bd):
    """Every head attends to one row at a random position (out = that V row at full magnitude: a row lost, doubled or
    weighted for the wrong head shows), and logits far apart between the splits of the context."""
    rng = np.random.default_rng(31)
    for b, hq, hkv, d, n in ((4, 32, 8, 128, 938), (1, 32, 8, 128, 3584), (2, 8, 8, 64, 700), (1, 16, 2, 128, 20000)):
        log("decode one key", (b, hq, hkv, d, n))
        kc = rng.standard_normal((b, hkv, n, d)).astype(np.float32)
        vc = rng.standard_normal((b, hkv, n, d)).astype(np.float32)
        pick = rng.integers(0, n, (b, hq))
        q = np.stack([np.stack([3.0 * kc[bi, h // (hq // hkv), pick[bi, h]] for h in range(hq)]) for bi in range(b)])
        q, kc, vc = (wl.quantize(x, "bf16")[0] for x in (q, kc, vc))
        out = to_host(bd.civic_decode_attn(to_dev(q), to_dev(kc), to_dev(vc), n))
        ref = oracle.decode_attention(widen(q), widen(kc), widen(vc), n)
        got = widen(out).astype(np.float64)
        assert np.abs(ref).mean() > 0.5 and np.abs(got - ref).max() <= attn_tol(ref, "bf16")
    # logits that grow along the context: the last split holds everything that matters, the first ones underflow
    b, hq, hkv, d, n = 1, 8, 2, 128, 2000
    q = rng.standard_normal((b, hq, d)).astype(np.float32)
    q[..., 0] = 8.0
    kc = rng.standard_normal((b, hkv, n, d)).astype(np.float32)
    kc[..., 0] = np.arange(n, dtype=np.float32)[None, None, :] * 2.0
    vc = rng.standard_normal((b, hkv, n, d)).astype(np.float32)
    q, kc, vc = (wl.quantize(x, "bf16")[0] for x in (q, kc, vc))
    check_decode(bd, q, kc, vc, n, "bf16")
    kc2 = widen(kc).copy()
    kc2[..., 0] = -kc2[..., 0]
    check_decode(bd, q, wl.quantize(kc2, "bf16")[0], vc, n, "bf16")


def test_decode_random_shapes(bd):
    rng = np.random.default_rng(777)
    worst = 0.0
    for it in range(200):
        d = int(rng.choice([32, 64, 72, 96, 128, 128, 256]))
        hkv = int(rng.choice([1, 2, 3, 8]))
        hq = hkv * int(rng.choice([1, 2, 3, 4, 4, 5, 8, 16]))
        b = int(rng.choice([1, 2, 5]))
        n = int(rng.choice([1, 2, 31, 32, 33, 127, 128, 129, 255, 300, 938, 1025, int(rng.integers(1, 3000))]))
        s_max = n + int(rng.integers(0, 9))
        dtype = "bf16" if rng.random() < 0.8 else "fp32"
        if dtype == "fp32" and d > 256:
            continue
        amp = float(rng.choice([0.5, 1.0, 3.0]))
        q = wl.quantize((rng.standard_normal((b, hq, d)) * amp).astype(np.float32), dtype)[0]
        kc = wl.quantize((rng.standard_normal((b, hkv, s_max, d)) * amp).astype(np.float32), dtype)[0]
        vc = wl.quantize(rng.standard_normal((b, hkv, s_max, d)).astype(np.float32), dtype)[0]
        if it % 40 == 0:
            log("decode random", it, (b, hq, hkv, d, s_max, n), dtype)
        out = to_host(bd.civic_decode_attn(to_dev(q), to_dev(kc), to_dev(vc), n))
        ref = oracle.decode_attention(widen(q), widen(kc), widen(vc), n)
        got = widen(out).astype(np.float64)
        err, tol = float(np.abs(got - ref).max()), attn_tol(ref, dtype)
        worst = max(worst, err / tol)
        assert np.isfinite(got).all() and err <= tol, ((b, hq, hkv, d, s_max, n), dtype, err, tol)
    log("   worst error / tolerance", worst)
