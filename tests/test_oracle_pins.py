"""Pins for the fp64 oracle: every check here is fixed by mathematics or by a
library routine, never by the oracle's own formula retyped.

(a) dense block-causal mask brute force      (b) single block == library SDPA
(c) incremental loop == one masked recompute (d) row sums and permutation invariance
plus closed forms, shift / duplication invariances, the two-segment
log-sum-exp merge, the ring's resident set and byte-exact commit.
"""
import collections
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand(rng, *shape):
    return rng.standard_normal(shape)


def dense_masked_attention(Q, K, V, blk_of, window_blocks=None):
    """Brute force: one N x N additive mask over the concatenation of all blocks.

    Token i sees token j iff blk(j) <= blk(i) and (with a ring of
    ``window_blocks`` cached blocks) blk(j) >= blk(i) - window_blocks.
    """
    N, H, D = Q.shape
    bi = blk_of[:, None]
    bj = blk_of[None, :]
    visible = bj <= bi
    if window_blocks is not None:
        visible &= bj >= bi - window_blocks
    add = np.where(visible, 0.0, -np.inf)
    out = np.zeros_like(Q)
    for h in range(H):
        logits = (Q[:, h, :] @ K[:, h, :].T) / math.sqrt(D) + add
        w = np.exp(logits - logits.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ V[:, h, :]
    return out


def run_incremental(Q, K, V, B, n, cap_blocks):
    """The generate-and-cache loop on the oracle: attention, then commit."""
    cache = oracle.BlockCacheOracle(cap_blocks)
    outs = []
    for b in range(B):
        sl = slice(b * n, (b + 1) * n)
        kc, vc = cache.logical()
        o, _ = oracle.attention(Q[sl], kc, vc, K[sl], V[sl])
        outs.append(o)
        cache.commit(K[sl], V[sl])
    return np.concatenate(outs, axis=0)


@pytest.mark.parametrize("B,n,H,D", [(3, 5, 2, 8), (4, 4, 3, 16), (1, 7, 1, 4)])
def test_a_dense_mask_bruteforce(B, n, H, D):
    rng = np.random.default_rng(10 + B)
    N = B * n
    Q, K, V = rand(rng, N, H, D), rand(rng, N, H, D), rand(rng, N, H, D)
    blk = np.repeat(np.arange(B), n)
    want = dense_masked_attention(Q, K, V, blk)
    got = run_incremental(Q, K, V, B, n, cap_blocks=B)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("cap", [1, 2, 3])
def test_a_dense_mask_with_ring_window(cap):
    B, n, H, D = 7, 4, 2, 8
    rng = np.random.default_rng(20 + cap)
    N = B * n
    Q, K, V = rand(rng, N, H, D), rand(rng, N, H, D), rand(rng, N, H, D)
    blk = np.repeat(np.arange(B), n)
    want = dense_masked_attention(Q, K, V, blk, window_blocks=cap)
    got = run_incremental(Q, K, V, B, n, cap_blocks=cap)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_b_single_block_is_plain_bidirectional_attention():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    n, H, D = 13, 3, 16
    q, k, v = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    got, _ = oracle.attention(q, None, None, k, v)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in (q, k, v))  # [1,H,n,D]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_b_cache_plus_block_is_library_cross_attention():
    """Queries over (cache ++ block) keys equals library SDPA with the concatenated K/V."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    n, C, H, D = 6, 11, 2, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    got, _ = oracle.attention(q, kc, vc, kb, vb)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.concatenate([kc, kb])).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.concatenate([vc, vb])).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_c_incremental_equals_recompute_from_scratch():
    """Loop {attention; commit} == for each block, attention with all earlier tokens as cache."""
    rng = np.random.default_rng(3)
    B, n, H, D = 4, 6, 2, 8
    N = B * n
    Q, K, V = rand(rng, N, H, D), rand(rng, N, H, D), rand(rng, N, H, D)
    inc = run_incremental(Q, K, V, B, n, cap_blocks=B)
    # recompute: the last block attends over the whole prefix at once, no cache object involved
    for b in range(B):
        sl = slice(b * n, (b + 1) * n)
        o, _ = oracle.attention(Q[sl], K[: b * n], V[: b * n], K[sl], V[sl])
        np.testing.assert_allclose(inc[sl], o, rtol=0, atol=1e-13)
    want = dense_masked_attention(Q, K, V, np.repeat(np.arange(B), n))
    np.testing.assert_allclose(inc, want, rtol=0, atol=1e-12)


def test_d_row_sums_and_lse():
    scipy_special = pytest.importorskip("scipy.special")
    rng = np.random.default_rng(4)
    n, C, H, D = 5, 9, 2, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    _, lse = oracle.attention(q, kc, vc, kb, vb)
    kall = np.concatenate([kc, kb])
    s = np.einsum("ihd,jhd->ihj", q, kall) / math.sqrt(D)
    np.testing.assert_allclose(lse, scipy_special.logsumexp(s, axis=-1), rtol=0, atol=1e-12)
    # probabilities implied by the oracle's normaliser sum to one
    p = np.exp(s - lse[..., None])
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-12)
    # with V = identity-like one-hot rows the output IS the probability row
    Lk = C + n
    Dv = Lk
    qpad = np.zeros((n, H, Dv)); qpad[..., :D] = q
    kpad = np.zeros((Lk, H, Dv)); kpad[..., :D] = kall
    eye = np.broadcast_to(np.eye(Lk)[:, None, :], (Lk, H, Dv)).copy()
    o, _ = oracle.attention(qpad, kpad[:C], eye[:C], kpad[C:], eye[C:], scale=1 / math.sqrt(D))
    np.testing.assert_allclose(o.sum(-1), 1.0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(o, p, rtol=0, atol=1e-12)


def test_d_permutation_of_cached_rows():
    rng = np.random.default_rng(5)
    n, C, H, D = 4, 12, 2, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    base, _ = oracle.attention(q, kc, vc, kb, vb)
    perm = rng.permutation(C)
    o, _ = oracle.attention(q, kc[perm], vc[perm], kb, vb)
    np.testing.assert_allclose(o, base, rtol=0, atol=1e-13)
    # permuting K without V must change the result (the pin has teeth)
    o2, _ = oracle.attention(q, kc[perm], vc, kb, vb)
    assert np.abs(o2 - base).max() > 1e-3


def test_golden_two_key_example():
    vals = {}
    with open(os.path.join(GOLDEN, "two_key_closed_form.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *xs = line.split()
            sym = {"LN3": math.log(3), "LN4": math.log(4)}
            vals[name] = np.array([sym[x] if x in sym else float(x) for x in xs])
    q = vals["q"].reshape(1, 1, 4)
    out, lse = oracle.attention(q, vals["k0"].reshape(1, 1, 4), vals["v0"].reshape(1, 1, 4),
                                vals["k1"].reshape(1, 1, 4), vals["v1"].reshape(1, 1, 4))
    np.testing.assert_allclose(out.reshape(4), vals["out"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse.reshape(1), vals["lse"], rtol=0, atol=1e-14)


def test_closed_form_identical_keys_give_mean_of_values():
    rng = np.random.default_rng(6)
    n, C, H, D = 3, 5, 2, 8
    q = rand(rng, n, H, D)
    key = rand(rng, 1, H, D)
    kc, kb = np.repeat(key, C, 0), np.repeat(key, n, 0)
    vc, vb = rand(rng, C, H, D), rand(rng, n, H, D)
    o, _ = oracle.attention(q, kc, vc, kb, vb)
    mean = np.concatenate([vc, vb]).mean(0)
    np.testing.assert_allclose(o, np.broadcast_to(mean, o.shape), rtol=0, atol=1e-13)


def test_closed_form_constant_values():
    rng = np.random.default_rng(7)
    n, C, H, D = 3, 5, 2, 8
    q, kb, kc = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, C, H, D)
    c = rand(rng, 1, H, D)
    o, _ = oracle.attention(q, kc, np.repeat(c, C, 0), kb, np.repeat(c, n, 0))
    np.testing.assert_allclose(o, np.broadcast_to(c, o.shape), rtol=0, atol=1e-13)


def test_closed_form_single_key():
    rng = np.random.default_rng(8)
    q, k, v = rand(rng, 1, 2, 8), rand(rng, 1, 2, 8), rand(rng, 1, 2, 8)
    o, lse = oracle.attention(q, None, None, k, v)
    np.testing.assert_array_equal(o, v)
    np.testing.assert_allclose(lse, np.einsum("ihd,ihd->ih", q, k) / math.sqrt(8), atol=1e-14)


@pytest.mark.parametrize("where", ["cache", "block"])
def test_closed_form_one_hot_limit(where):
    rng = np.random.default_rng(9)
    n, C, H, D = 3, 6, 1, 4
    kc, vc = 0.01 * rand(rng, C, H, D), rand(rng, C, H, D)
    kb, vb = 0.01 * rand(rng, n, H, D), rand(rng, n, H, D)
    q = np.zeros((n, H, D)); q[..., 0] = 1.0
    if where == "cache":
        kc[2, 0, 0] = 120.0  # scaled score +60 above the rest
        target = vc[2]
    else:
        kb[1, 0, 0] = 120.0
        target = vb[1]
    o, _ = oracle.attention(q, kc, vc, kb, vb)
    np.testing.assert_allclose(o, np.broadcast_to(target, o.shape), rtol=0, atol=1e-20 + 1e-12)


def test_invariance_common_key_shift():
    rng = np.random.default_rng(11)
    n, C, H, D = 4, 7, 2, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    base, lse0 = oracle.attention(q, kc, vc, kb, vb)
    shift = rand(rng, 1, H, D)
    o, lse1 = oracle.attention(q, kc + shift, vc, kb + shift, vb)
    np.testing.assert_allclose(o, base, rtol=0, atol=1e-12)
    # the normaliser moves by exactly the per-row constant
    np.testing.assert_allclose(lse1 - lse0, np.einsum("ihd,hd->ih", q, shift[0]) / math.sqrt(D), atol=1e-12)


def test_invariance_duplicated_keys():
    rng = np.random.default_rng(12)
    n, C, H, D = 4, 6, 2, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    # all keys live in the "cache" slot here; block holds one copy, cache the other copy plus itself
    kall, vall = np.concatenate([kc, kb]), np.concatenate([vc, vb])
    base, lse0 = oracle.attention(q, kc, vc, kb, vb)
    o, lse1 = oracle.attention(q, np.concatenate([kall, kc]), np.concatenate([vall, vc]), kb, vb)
    np.testing.assert_allclose(o, base, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse1 - lse0, math.log(2.0), rtol=0, atol=1e-12)


def test_identity_two_segment_lse_merge():
    """Attention over cache++block == LSE-weighted mix of attention over each alone."""
    rng = np.random.default_rng(13)
    n, C, H, D = 4, 9, 2, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    full, lse = oracle.attention(q, kc, vc, kb, vb)
    ob, lb = oracle.attention(q, None, None, kb, vb)
    # "cache alone": queries against the cache tokens only == single-key-set attention
    rows = np.repeat(np.arange(n), H); heads = np.tile(np.arange(H), n)
    # use the cache rows as the block of a (n_c = C) problem with queries padded: do it per row via numpy
    s = np.einsum("ihd,jhd->ihj", q, kc) / math.sqrt(D)
    lc = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    pc = np.exp(s - lc[..., None])
    oc = np.einsum("ihj,jhd->ihd", pc, vc)
    wb = np.exp(lb - lse)[..., None]
    wc = np.exp(lc - lse)[..., None]
    np.testing.assert_allclose(wb + wc, 1.0, atol=1e-12)
    np.testing.assert_allclose(wc * oc + wb * ob, full, rtol=0, atol=1e-12)


def test_merge_equals_attention_over_the_union():
    """oracle.merge of attention over two disjoint key subsets == attention over their union
    (itself pinned by the brute-force and library pins), for outputs and log-sum-exp; in either order."""
    rng = np.random.default_rng(21)
    n, H, D = 5, 3, 8
    q = rand(rng, n, H, D)
    ka, va = rand(rng, 7, H, D), rand(rng, 7, H, D)
    kb, vb = rand(rng, 11, H, D) * 3.0, rand(rng, 11, H, D)
    kblk, vblk = rand(rng, n, H, D), rand(rng, n, H, D)
    full, lse = oracle.attention(q, np.concatenate([ka, kb]), np.concatenate([va, vb]), None, None)
    oa, la = oracle.attention(q, ka, va, None, None)
    ob, lb = oracle.attention(q, kb, vb, None, None)
    for (o1, l1, o2, l2) in ((oa, la, ob, lb), (ob, lb, oa, la)):
        om, lm = oracle.merge(o1, l1, o2, l2)
        np.testing.assert_allclose(om, full, rtol=0, atol=1e-13)
        np.testing.assert_allclose(lm, lse, rtol=0, atol=1e-13)
    # cache part + the block alone == cache and block together
    full, lse = oracle.attention(q, ka, va, kblk, vblk)
    oblk, lblk = oracle.attention(q, None, None, kblk, vblk)
    om, lm = oracle.merge(oa, la, oblk, lblk)
    np.testing.assert_allclose(om, full, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lm, lse, rtol=0, atol=1e-13)


def test_cache_only_key_set_is_library_cross_attention():
    """Without a current block the oracle is plain cross attention of q over the given keys."""
    import torch
    rng = np.random.default_rng(24)
    n, C, H, D = 4, 9, 2, 8
    q, kc, vc = rand(rng, n, H, D), rand(rng, C, H, D), rand(rng, C, H, D)
    got, _ = oracle.attention(q, kc, vc, None, None)
    t = lambda a: torch.from_numpy(a).permute(1, 0, 2)
    want = torch.nn.functional.scaled_dot_product_attention(t(q), t(kc), t(vc)).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    with pytest.raises(Exception):
        oracle.attention(q, None, None, None, None)


def test_merge_weights_are_the_softmax_of_the_two_lse():
    """The mixing weights must be softmax([lse_a, lse_b]) and the new lse their logsumexp (scipy)."""
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(22)
    la, lb = rng.standard_normal((4, 2)) * 30.0, rng.standard_normal((4, 2)) * 30.0  # far apart: no overflow allowed
    oa, ob = rand(rng, 4, 2, 6), rand(rng, 4, 2, 6)
    om, lm = oracle.merge(oa, la, ob, lb)
    w = softmax(np.stack([la, lb], -1), axis=-1)
    np.testing.assert_allclose(om, w[..., 0:1] * oa + w[..., 1:2] * ob, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(lm, logsumexp(np.stack([la, lb], -1), axis=-1), rtol=1e-14, atol=1e-13)
    assert np.isfinite(om).all() and np.isfinite(lm).all()


def test_merge_closed_forms():
    rng = np.random.default_rng(23)
    oa, ob = rand(rng, 3, 2, 4), rand(rng, 3, 2, 4)
    l = rng.standard_normal((3, 2))
    om, lm = oracle.merge(oa, l, ob, l)  # equal weight: the mean, lse + ln 2
    np.testing.assert_allclose(om, 0.5 * (oa + ob), atol=1e-15)
    np.testing.assert_allclose(lm, l + math.log(2.0), atol=1e-15)
    om, lm = oracle.merge(oa, l, ob, np.full_like(l, -np.inf))  # an empty key set changes nothing
    np.testing.assert_allclose(om, oa, atol=0)
    np.testing.assert_allclose(lm, l, atol=0)
    om, lm = oracle.merge(oa, l, ob, l - 800.0)  # a hopelessly small one neither
    np.testing.assert_allclose(om, oa, atol=1e-300)


def test_block_range_selection_of_the_cache_oracle():
    """logical(ranges) returns exactly the named resident blocks, oldest first (checked against
    block contents that encode their own ordinal)."""
    cache = oracle.BlockCacheOracle(4)
    for b in range(7):  # residents: ordinals 3, 4, 5, 6
        cache.commit(np.full((2, 1, 1), float(b)), np.full((2, 1, 1), float(-b)))
    k, v = cache.logical([(0, 1), (2, 2)])
    assert k[:, 0, 0].tolist() == [3, 3, 5, 5, 6, 6] and v[:, 0, 0].tolist() == [-3, -3, -5, -5, -6, -6]
    k, _ = cache.logical([(1, 3)])
    assert k[:, 0, 0].tolist() == [4, 4, 5, 5, 6, 6]
    assert cache.logical([]) == (None, None) and cache.logical([(2, 0)]) == (None, None)
    with pytest.raises(IndexError):
        cache.logical([(2, 3)])


def test_growing_the_cache_oracle_keeps_blocks_and_delays_eviction():
    """After grow() the resident blocks are the same ones in the same order, commits evict nothing
    until the larger window is full, and from then on the oldest block again (checked against the
    list of everything committed, sliced by hand)."""
    cache = oracle.BlockCacheOracle(3)
    for b in range(5):  # residents: 2, 3, 4
        cache.commit(np.full((1, 1, 1), float(b)), np.full((1, 1, 1), float(b)))
    cache.grow(5)
    assert cache.ordinals == [2, 3, 4] and cache.committed == 5
    for b in range(5, 11):
        cache.commit(np.full((1, 1, 1), float(b)), np.full((1, 1, 1), float(b)))
        everything = list(range(2, b + 1))  # 0 and 1 were gone before the grow
        assert cache.ordinals == everything[-5:]
        assert cache.logical()[0][:, 0, 0].tolist() == [float(o) for o in everything[-5:]]
    with pytest.raises(ValueError):
        cache.grow(5)


def test_block_list_selection_of_the_cache_oracle():
    """logical(blocks=...) returns the listed resident blocks in the list's order."""
    cache = oracle.BlockCacheOracle(4)
    for b in range(7):  # residents: ordinals 3, 4, 5, 6
        cache.commit(np.full((2, 1, 1), float(b)), np.full((2, 1, 1), float(-b)))
    k, v = cache.logical(blocks=[3, 0, 2])
    assert k[:, 0, 0].tolist() == [6, 6, 3, 3, 5, 5] and v[:, 0, 0].tolist() == [-6, -6, -3, -3, -5, -5]
    assert cache.logical(blocks=[]) == (None, None)
    for bad in ([4], [-1], [1, 1]):
        with pytest.raises(IndexError):
            cache.logical(blocks=bad)


def test_block_list_attention_equals_a_block_sparse_dense_mask():
    """Attention of the last block over a chosen subset of earlier blocks plus itself equals one
    dense N x N computation with the other blocks' columns masked out (KV Management section:
    selective fetch of cached blocks), whatever the order of the list."""
    rng = np.random.default_rng(21)
    B, n, H, D = 6, 4, 2, 8
    N = B * n
    Q, K, V = rand(rng, N, H, D), rand(rng, N, H, D), rand(rng, N, H, D)
    cache = oracle.BlockCacheOracle(B)
    for b in range(B - 1):
        cache.commit(K[b * n:(b + 1) * n], V[b * n:(b + 1) * n])
    last = slice((B - 1) * n, N)
    for picks in ([0, 2, 3], [4, 1], [3, 0, 2, 1, 4], []):
        visible = np.zeros(N, dtype=bool)
        visible[last] = True
        for b in picks:
            visible[b * n:(b + 1) * n] = True
        want = np.zeros((n, H, D))
        for h in range(H):
            logits = (Q[last, h, :] @ K[:, h, :].T) / math.sqrt(D) + np.where(visible, 0.0, -np.inf)[None, :]
            w = np.exp(logits - logits.max(axis=1, keepdims=True))
            want[:, h, :] = (w / w.sum(axis=1, keepdims=True)) @ V[:, h, :]
        kc, vc = cache.logical(blocks=picks)
        got, _ = oracle.attention(Q[last], kc, vc, K[last], V[last])
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_scale_default_is_inverse_sqrt_head_dim():
    rng = np.random.default_rng(14)
    n, H, D = 3, 1, 16
    q, k, v = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    a, _ = oracle.attention(q, None, None, k, v)
    b, _ = oracle.attention(q * 0.25, None, None, k, v, scale=1.0)  # 1/sqrt(16) folded into q
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_selected_rows_match_full():
    rng = np.random.default_rng(15)
    n, C, H, D = 9, 5, 3, 8
    q, kb, vb = rand(rng, n, H, D), rand(rng, n, H, D), rand(rng, n, H, D)
    kc, vc = rand(rng, C, H, D), rand(rng, C, H, D)
    full, lse = oracle.attention(q, kc, vc, kb, vb)
    rows = np.array([8, 0, 3, 3]); heads = np.array([2, 1, 0, 2])
    o, l = oracle.attention_rows(q, kc, vc, kb, vb, rows, heads)
    np.testing.assert_array_equal(o, full[rows, heads])
    np.testing.assert_array_equal(l, lse[rows, heads])


def test_rejects_bad_selection():
    q = np.zeros((2, 1, 4))
    with pytest.raises(RuntimeError):
        oracle.attention_rows(q, None, None, q, q, [2], [0])
    with pytest.raises(RuntimeError):
        oracle.attention_rows(q, None, None, q, q, [0], [1])


# ---- the block cache (ring) ----

@pytest.mark.parametrize("cap", [1, 3, 7])
def test_ring_resident_set(cap):
    """After t commits the resident blocks are ordinals max(0, t-cap) .. t-1, oldest first."""
    cache = oracle.BlockCacheOracle(cap)
    for t in range(1, 45):
        blk = np.full((2, 1, 4), t - 1, dtype=np.float32)
        cache.commit(blk, -blk)
        assert cache.committed == t
        assert cache.ordinals == list(range(max(0, t - cap), t))
        k, v = cache.logical()
        assert k.shape[0] == 2 * min(t, cap)
        np.testing.assert_array_equal(k[::2, 0, 0], np.arange(max(0, t - cap), t))
        np.testing.assert_array_equal(v, -k)


def test_commit_is_a_byte_exact_copy_and_owns_its_data():
    rng = np.random.default_rng(16)
    bits = rng.integers(0, 1 << 16, size=(8, 2, 4), dtype=np.uint16)
    # force special patterns: NaN payloads, -0.0, denormals, infinities (bf16 bit patterns)
    bits.flat[:6] = [0x7FC1, 0xFFFF, 0x8000, 0x0001, 0x7F80, 0xFF80]
    cache = oracle.BlockCacheOracle(2)
    kb = bits.copy(); vb = (bits ^ 0x5555).astype(np.uint16)
    cache.commit(kb, vb)
    kb[:] = 0  # caller's buffer is reused afterwards
    k, v = cache.logical()
    assert k.tobytes() == bits.tobytes()
    assert v.tobytes() == (bits ^ 0x5555).astype(np.uint16).tobytes()


def test_bf16_widening_is_exact():
    torch = pytest.importorskip("torch")
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.bf16_bits_to_f64(bits)
    np.testing.assert_array_equal(got[finite], t[finite])


# ---- fp8 (E4M3) cache variant: the format and the commit's rounding rule ----------------------

def test_e4m3_widening_all_256_codes_against_torch():
    """oracle.e4m3_bits_to_f64 (the format's definition written out) against the library's own
    float8_e4m3fn -> float64 conversion, for every code."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.e4m3_bits_to_f64(codes)
    want = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    assert np.signbit(got[0x80]) and got[0x80] == 0  # -0
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6 and got[0x38] == 1.0
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF])
    # every E4M3 value is a bfloat16 value (attention reads the cache through bf16 operands)
    f = got[~np.isnan(got)]
    assert np.array_equal(f, f.astype(np.float32).view(np.uint32).__and__(0xFFFF0000).view(np.float32).astype(np.float64))


def test_e4m3_rounding_of_every_bf16_value_against_torch():
    """oracle.quantize_e4m3 on all 65536 bfloat16 patterns against the library's round-to-nearest-
    even conversion wherever that one stays finite (|x| <= 464: the library rounds as if the code
    after 448, which the format gives to NaN, were the value 480, so everything nearer to 480 than
    to 448 becomes NaN there); beyond it the commit's rule saturates at 448."""
    import torch
    bits = np.arange(65536, dtype=np.uint16)
    x = oracle.bf16_bits_to_f64(bits)
    got = oracle.quantize_e4m3(x)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    want = t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    inside = np.abs(x) <= 464.0
    assert inside.sum() > 30000
    assert np.array_equal(got[inside], want[inside])
    # saturation and NaN
    big = np.abs(x) > 464.0
    assert np.array_equal(got[big] & 0x7F, np.full(big.sum(), 0x7E, dtype=np.uint8))
    assert np.array_equal((got[big] & 0x80) != 0, np.signbit(x[big]))
    assert np.all((got[np.isnan(x)] & 0x7F) == 0x7F)


def test_e4m3_rounding_closed_forms():
    """Exact values map to their own code; ties go to the even code; the subnormal range; saturation."""
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    assert np.array_equal(oracle.quantize_e4m3(oracle.e4m3_bits_to_f64(codes)), codes)
    q = lambda v: int(oracle.quantize_e4m3(np.array([v]))[0])
    assert q(1.0625) == 0x38 and q(1.1875) == 0x3A  # halfway 1.0 | 1.125 -> even code; halfway 1.125 | 1.25 -> even code
    assert q(1.0626) == 0x39 and q(1.0624) == 0x38
    assert q(2.0 ** -10) == 0x00 and q(3 * 2.0 ** -10) == 0x02 and q(2.0 ** -10 * 1.001) == 0x01
    assert q(-2.0 ** -10) == 0x80
    assert q(464.0) == 0x7E and q(1e6) == 0x7E and q(-np.inf) == 0xFE and q(np.inf) == 0x7E
    assert q(447.0) == 0x7E and q(432.0) == 0x7E and q(431.9) == 0x7D  # halfway 416 | 448 -> even code 0x7E
    # the round trip through bf16 bit patterns
    bits = np.array([0x3F80, 0x3F88, 0xBF98, 0x7F80, 0x7FC0, 0x0001], dtype=np.uint16)  # 1, 1.0625, -1.1875, inf, nan, denormal
    out = oracle.bf16_bits_through_e4m3(bits)
    assert list(out[:4]) == [0x3F80, 0x3F80, 0xBFA0, 0x43E0] and out[5] == 0 and (out[4] & 0x7FFF) > 0x7F80
