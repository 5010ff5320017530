"""GPU tests of the boundary's corners: a softmax scale other than the default, values
that are not finite or overflow the key-norm bound, and canary rows behind every output
buffer (nothing may be written past the end of out, lse, k_out or v_out)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import TORCH_DTYPE, OracleCacheF, assert_attention_close, to_np_exact

pytestmark = pytest.mark.gpu

LSE_TOL = {ifx.IFX_F32: 2e-5, ifx.IFX_BF16: 2e-3}


def all_pairs(n, H):
    return np.repeat(np.arange(n), H), np.tile(np.arange(H), n)


@pytest.mark.parametrize("dtype,D", [(ifx.IFX_BF16, 128), (ifx.IFX_F32, 64)])
@pytest.mark.parametrize("scale", [0.05, 0.25])
def test_softmax_scale_other_than_default(gpu_device, dtype, D, scale):
    """ifx_kv_cache_configure's softmax_scale reaches the scores, the norm bound and the
    log-sum-exp.  0.05 is below 1/sqrt(D) (flatter rows); 0.25 is above it: with RMS-normed bf16
    rows the bound is 128 * 0.25 * log2(e) = 46 (still the fixed-maximum variant), and the
    rows with 1.5 x longer queries go over the limit and take the running maximum."""
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    n, H, cap = 200, 3, 3
    with ifx.KVCache(1, H, D, cap * n, n, dtype, softmax_scale=scale) as cache:
        oc = OracleCacheF(cap, tdtype)
        for b in range(cap + 1):  # wraps once
            _, k, v = synth.draw_qkv(83, b, 0, 0, n, H, D, tdtype, dev, True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(83, 50, 0, 0, n, H, D, tdtype, dev, True)
        q = q.clone()
        q[64:128] *= 1.5  # exact in bf16
        out = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        lse = torch.full((n, H), float("nan"), dtype=torch.float32, device=dev)
        cache.attention_blocks(0, q, k, v, None, out, lse)
        out2 = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        cache.attention(0, q, k, v, out2)
        torch.cuda.synchronize()
        rows, heads = all_pairs(n, H)
        kc, vc = oc.logical()
        want, want_lse = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v),
                                               rows, heads, scale=scale)
        # a wrong scale is far outside the tolerance: the default 1/sqrt(D) must not pass here
        wrong, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        assert np.abs(wrong - want).max() > 10 * (2e-2 if dtype == ifx.IFX_BF16 else 1e-5)
        gain = max(1.0, scale * np.sqrt(D))
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, f"scale {scale}", input_scale=gain)
        assert synth.raw_bytes(out) == synth.raw_bytes(out2)
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[dtype] * gain


def test_bf16_key_norm_overflow_and_zero_query(gpu_device):
    """Finite inputs that break the norm bound: a cached key whose squared norm overflows fp32
    (elements 2^66; head 0's queries are scaled by 2^-47 so that the scores themselves stay
    within fp32's accurate range) and a query row of zeros.  The bound is inf for ordinary rows
    and 0 * inf for the zero row; both must send the wavefront to the running maximum, where the
    zero row gives the mean of V and the other rows of that head are one-hot on the huge key or
    ignore it.  Head 1 has no such key and stays on the fixed maximum."""
    dev = gpu_device
    n, H, D, cap = 72, 2, 128, 2
    with ifx.KVCache(1, H, D, cap * n, n, ifx.IFX_BF16) as cache:
        oc = OracleCacheF(cap, torch.bfloat16)
        for b in range(cap):
            _, k, v = synth.draw_qkv(89, b, 0, 0, n, H, D, torch.bfloat16, dev, True)
            if b == 0:
                k = k.clone()
                k[5, 0, :] = torch.tensor(2.0 ** 66) * torch.sign(k[5, 0, :].float()).to(torch.bfloat16)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(89, 9, 0, 0, n, H, D, torch.bfloat16, dev, True)
        q = q.clone()
        q[:, 0, :] *= 2.0 ** -47  # exact
        q[3, 0, :] = 0
        q[40, 1, :] = 0
        out = torch.full((n, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        rows, heads = all_pairs(n, H)
        kc, vc = oc.logical()
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        assert np.isfinite(want).all()
        got = to_np_exact(out)[rows, heads].astype(np.float64)
        assert_attention_close(got, want, ifx.IFX_BF16, "huge key, zero query", input_scale=8.0)
        # the zero rows are the mean of all V rows of their head
        vall = np.concatenate([vc, synth.to_f64_numpy(v)])
        assert np.abs(to_np_exact(out)[3, 0] - vall[:, 0].mean(0)).max() <= 2e-3
        assert np.abs(to_np_exact(out)[40, 1] - vall[:, 1].mean(0)).max() <= 2e-3


def test_bf16_non_finite_inputs_stay_in_their_head(gpu_device):
    """Values that are not finite are not detected (include/ifx.h): the call succeeds, writes all
    of out, and the heads that hold none of them are as exact as ever.  An infinite cached key, a
    NaN in the current block's V and a NaN query, each in head 0; head 1 must match the oracle."""
    dev = gpu_device
    n, H, D, cap = 136, 2, 128, 2
    for case in ("inf cached key", "nan block v", "nan query"):
        with ifx.KVCache(1, H, D, cap * n, n, ifx.IFX_BF16) as cache:
            oc = OracleCacheF(cap, torch.bfloat16)
            for b in range(cap):
                _, k, v = synth.draw_qkv(97, b, 0, 0, n, H, D, torch.bfloat16, dev, True)
                if case == "inf cached key" and b == 1:
                    k = k.clone()
                    k[7, 0, 3] = float("inf")
                cache.commit(0, k, v)
                oc.commit(k, v)
            q, k, v = synth.draw_qkv(97, 9, 0, 0, n, H, D, torch.bfloat16, dev, True)
            q, v = q.clone(), v.clone()
            if case == "nan block v":
                v[100, 0, 64] = float("nan")
            if case == "nan query":
                q[20, 0, 1] = float("nan")
            out = torch.full((n + 1, H, D), 7.0, dtype=torch.bfloat16, device=dev)
            cache.attention(0, q, k, v, out[:n])
            torch.cuda.synchronize()
            assert (out[n] == 7.0).all(), case
            rows, heads = np.arange(n), np.ones(n, dtype=np.int64)
            kc, vc = oc.logical()
            # the oracle is given head 1 only in finite company: replace head 0 by zeros
            def h1(a):
                a = a.copy()
                a[:, 0] = 0
                return a
            want, _ = oracle.attention_rows(h1(synth.to_f64_numpy(q)), h1(kc), h1(vc), h1(synth.to_f64_numpy(k)),
                                            h1(synth.to_f64_numpy(v)), rows, heads)
            assert_attention_close(to_np_exact(out[:n])[rows, heads].astype(np.float64), want, ifx.IFX_BF16, case)
            if case == "nan query":  # rows of head 0 that hold no NaN themselves are untouched by it
                rows0 = np.array([r for r in range(n) if r != 20])
                want0, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v),
                                                 rows0, np.zeros_like(rows0))
                assert_attention_close(to_np_exact(out[:n])[rows0, 0].astype(np.float64), want0, ifx.IFX_BF16, case + " head 0")


@pytest.mark.parametrize("dtype,D", [(ifx.IFX_BF16, 128), (ifx.IFX_F32, 64)])
def test_canary_rows_behind_every_output(gpu_device, dtype, D):
    """out, lse, k_out and v_out are followed by canary rows that every call must leave alone:
    ragged block (n = 200: the last query tile and the last key tile are partial), wrapped ring,
    plain, listed-block and merge calls, and the cache read-back."""
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    n, H, cap = 200, 3, 2
    with ifx.KVCache(1, H, D, cap * n, n, dtype) as cache:
        for b in range(cap + 1):
            _, k, v = synth.draw_qkv(101, b, 0, 0, n, H, D, tdtype, dev, True)
            cache.commit(0, k, v)
        q, k, v = synth.draw_qkv(101, 9, 0, 0, n, H, D, tdtype, dev, True)
        pad = 3
        def buf(rows, *shape):
            return torch.full((rows + pad, *shape), 5.0, dtype=tdtype if shape[-1] == D else torch.float32, device=dev)
        out, out_b = buf(n, H, D), buf(n, H, D)
        lse, lse_b = buf(n, H), buf(n, H)
        cache.attention(0, q, k, v, out[:n])
        cache.attention_blocks(0, q, k, v, [1], out_b[:n], lse_b[:n])
        cache.attention_blocks(0, q, None, None, [0], out[:n], lse[:n])
        ifx.ifx_attention_merge(out[:n], lse[:n], out_b[:n], lse_b[:n], out[:n], lse[:n], n * H, D, dtype)
        C = cache.len(0)
        k_out, v_out = buf(C, H, D), buf(C, H, D)
        cache.read(0, k_out[:C], v_out[:C], True)
        cache.read(0, k_out[:C], v_out[:C], False)
        torch.cuda.synchronize()
        for name, t, rows in (("out", out, n), ("out_b", out_b, n), ("lse", lse, n), ("lse_b", lse_b, n),
                              ("k_out", k_out, C), ("v_out", v_out, C)):
            assert (t[rows:] == 5.0).all(), name
            assert torch.isfinite(t[:rows].float()).all(), name
