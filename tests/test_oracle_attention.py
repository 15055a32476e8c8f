"""Pins for the oracle's exact attention, map reuse and map storage rounding.

Algorithm 2 (both branches) and the map equation of the paper's Sec. 4.  Nothing here is
computed by the GPU path: hand-worked values, closed forms, invariants and CPU library
routines (torch, fp64) only.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _rand(shape, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=torch.float64).float().numpy()


# ---------------------------------------------------------------- exact attention

def test_hand_worked_two_tokens(oracle_mod):
    # D = 1, scale = 1: logits of token 1 are [q1*k0, q1*k1] = [0, ln 3] -> P = [1/4, 3/4]
    Q = np.array([[[[1.0], [1.0]]]], np.float32)
    K = np.array([[[[0.0], [math.log(3.0)]]]], np.float32)
    V = np.array([[[[8.0], [4.0]]]], np.float32)
    O, P = oracle_mod.attention_exact(Q, K, V, causal=True, scale=1.0, return_map=True)
    k1 = float(np.float32(math.log(3.0)))
    p11 = math.exp(k1) / (1.0 + math.exp(k1))
    np.testing.assert_allclose(P[0, 0], [[1.0, 0.0], [1 - p11, p11]], rtol=0, atol=1e-15)
    np.testing.assert_allclose(O[0, 0, :, 0], [8.0, 8 * (1 - p11) + 4 * p11], rtol=0, atol=1e-14)
    assert abs(p11 - 0.75) < 1e-7
    # without the mask token 0 also sees token 1: logits [0, ln 3] again
    O2, P2 = oracle_mod.attention_exact(Q, K, V, causal=False, scale=1.0, return_map=True)
    np.testing.assert_allclose(P2[0, 0], [[1 - p11, p11], [1 - p11, p11]], atol=1e-15)


def test_default_scale_is_inverse_sqrt_head_dim(oracle_mod):
    # one query, two keys, D = 4: logits = <q,k>/2
    Q = np.zeros((1, 1, 2, 4), np.float32)
    K = np.zeros((1, 1, 2, 4), np.float32)
    Q[0, 0, 1] = [2, 0, 0, 0]
    K[0, 0, 0] = [1, 0, 0, 0]      # <q1,k0> = 2 -> logit 1
    K[0, 0, 1] = [3, 0, 0, 0]      # <q1,k1> = 6 -> logit 3
    V = np.array([[[[1, 0, 0, 0], [0, 1, 0, 0]]]], np.float32)
    _, P = oracle_mod.attention_exact(Q, K, V, return_map=True)
    e = math.exp(-2.0)
    np.testing.assert_allclose(P[0, 0, 1], [e / (1 + e), 1 / (1 + e)], atol=1e-15)


def test_map_invariants(oracle_mod):
    B, H, S, D = 2, 3, 37, 16
    Q, K, V = _rand((B, H, S, D), 10), _rand((B, H, S, D), 11), _rand((B, H, S, D), 12)
    _, P = oracle_mod.attention_exact(Q, K, V, causal=True, return_map=True)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-12)
    assert (P >= 0).all()
    iu = np.triu_indices(S, 1)
    assert (P[..., iu[0], iu[1]] == 0.0).all()          # exact zeros above the diagonal
    first = np.zeros(S); first[0] = 1.0
    assert (P[..., 0, :] == first).all()                # token 0 attends only to itself
    _, Pd = oracle_mod.attention_exact(Q, K, V, causal=False, return_map=True)
    np.testing.assert_allclose(Pd.sum(-1), 1.0, atol=1e-12)
    assert (Pd > 0).all()


def test_zero_queries_give_prefix_means(oracle_mod):
    B, H, S, D = 1, 2, 19, 8
    K, V = _rand((B, H, S, D), 13), _rand((B, H, S, D), 14)
    O, P = oracle_mod.attention_exact(np.zeros((B, H, S, D), np.float32), K, V, return_map=True)
    for i in range(S):
        np.testing.assert_allclose(P[0, 0, i, : i + 1], 1.0 / (i + 1), rtol=1e-15)
    prefix = np.cumsum(V.astype(np.float64), axis=2) / np.arange(1, S + 1)[None, None, :, None]
    np.testing.assert_allclose(O, prefix, rtol=1e-13, atol=1e-13)


def test_single_token_returns_v(oracle_mod):
    Q, K, V = _rand((3, 2, 1, 8), 15), _rand((3, 2, 1, 8), 16), _rand((3, 2, 1, 8), 17)
    O = oracle_mod.attention_exact(Q, K, V)
    assert np.array_equal(O, V.astype(np.float64))


def test_row_shift_invariance(oracle_mod):
    # adding one vector u to every key adds <q_i,u> to all logits of row i: the map is unchanged
    B, H, S, D = 1, 1, 23, 8
    Q, K, V = _rand((B, H, S, D), 18), _rand((B, H, S, D), 19), _rand((B, H, S, D), 20)
    K = np.round(K * 1024) / np.float32(1024)           # coarse grid: K + u is exact in fp32
    u = np.float32(0.5) * np.ones((D,), np.float32)
    _, P0 = oracle_mod.attention_exact(Q, K, V, return_map=True)
    _, P1 = oracle_mod.attention_exact(Q, K + u, V, return_map=True)
    np.testing.assert_allclose(P1, P0, rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_against_library_sdpa(oracle_mod, causal, hq, hkv):
    B, S, D = 2, 45, 24                                   # S != D: a transposed operand cannot pass
    Q, K, V = _rand((B, hq, S, D), 21), _rand((B, hkv, S, D), 22), _rand((B, hkv, S, D), 23)
    O = oracle_mod.attention_exact(Q, K, V, causal=causal)
    g = hq // hkv
    q, k, v = (torch.from_numpy(x).double() for x in (Q, K, V))
    ref = F.scaled_dot_product_attention(q, k.repeat_interleave(g, 1), v.repeat_interleave(g, 1),
                                         is_causal=causal)
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-11, atol=1e-12)
    O2 = oracle_mod.attention_exact(Q, K, V, causal=causal, scale=0.3)
    ref2 = F.scaled_dot_product_attention(q, k.repeat_interleave(g, 1), v.repeat_interleave(g, 1),
                                          is_causal=causal, scale=0.3)
    np.testing.assert_allclose(O2, ref2.numpy(), rtol=1e-11, atol=1e-12)


def test_row_sel_skips_served_items(oracle_mod):
    Q, K, V = _rand((3, 2, 9, 4), 24), _rand((3, 2, 9, 4), 25), _rand((3, 2, 9, 4), 26)
    full = oracle_mod.attention_exact(Q, K, V)
    out = np.full((3, 2, 9, 4), 7.0)
    oracle_mod.attention_exact(Q, K, V, row_sel=np.array([-1, 5, -1]), out=out)
    assert np.array_equal(out[0], full[0]) and np.array_equal(out[2], full[2])
    assert (out[1] == 7.0).all()


@pytest.mark.parametrize("causal", [True, False])
def test_key_lengths_against_library_mask(oracle_mod, causal):
    # a right-padded batch: keys at or beyond the sentence's length are hidden from every row
    B, H, S, D = 3, 2, 19, 8
    Q, K, V = _rand((B, H, S, D), 31), _rand((B, H, S, D), 32), _rand((B, H, S, D), 33)
    lens = np.array([19, 7, 1], np.int32)
    O, P = oracle_mod.attention_exact(Q, K, V, causal=causal, key_len=lens, return_map=True)
    q, k, v = (torch.from_numpy(x).double() for x in (Q, K, V))
    keep = torch.arange(S)[None, :] < torch.from_numpy(lens)[:, None]          # [B, S] keys
    mask = keep[:, None, None, :].expand(B, 1, S, S).clone()
    if causal:
        mask &= torch.ones(S, S, dtype=torch.bool).tril()
    ref = F.scaled_dot_product_attention(q, k, v, attn_mask=mask)
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-11, atol=1e-12)
    for b in range(B):
        assert (P[b, :, :, lens[b]:] == 0.0).all()                            # exact zeros on padding
        np.testing.assert_allclose(P[b].sum(-1), 1.0, rtol=1e-13)
    # what lies in the padding does not matter
    K2, V2 = K.copy(), V.copy()
    for b in range(B):
        K2[b, :, lens[b]:], V2[b, :, lens[b]:] = 1e3, -1e3
    O2 = oracle_mod.attention_exact(Q, K2, V2, causal=causal, key_len=lens)
    assert np.array_equal(O2, O)
    # a sentence of one token: every row returns V[0]
    np.testing.assert_allclose(O[2], np.broadcast_to(V[2, :, :1].astype(np.float64), O[2].shape),
                               rtol=1e-15)
    # the full length is the unpadded result
    full = oracle_mod.attention_exact(Q, K, V, causal=causal)
    assert np.array_equal(O[0], full[0])
    # causal rows inside the sentence never saw the padding anyway
    if causal:
        for b in range(B):
            assert np.array_equal(O[b, :, :lens[b]], full[b, :, :lens[b]])
    with pytest.raises(RuntimeError):
        oracle_mod.attention_exact(Q, K, V, key_len=np.array([19, 0, 1], np.int32))
    with pytest.raises(RuntimeError):
        oracle_mod.attention_exact(Q, K, V, key_len=np.array([20, 1, 1], np.int32))


# -------------------------------------------------------------------- map reuse

def test_identity_map_returns_v_exactly(oracle_mod):
    S, D = 12, 5
    maps = np.broadcast_to(np.eye(S, dtype=np.float32), (1, 1, 2, S, S)).copy()
    V = _rand((3, 1, 2, S, D), 30)
    O = oracle_mod.apply(maps, np.zeros(3, np.int32), V)
    assert np.array_equal(O, V.astype(np.float64))


def test_uniform_lower_triangular_map_gives_prefix_means(oracle_mod):
    S, D = 16, 4                     # 1/(i+1) is exact in fp32 only for powers of two: use fp64 check
    A = np.tril(np.ones((S, S))) / np.arange(1, S + 1)[:, None]
    maps = A.astype(np.float32).reshape(1, 1, 1, S, S)
    V = _rand((1, 1, 1, S, D), 31)
    O = oracle_mod.apply(maps, np.zeros(1, np.int32), V)
    ref = maps[0, 0, 0].astype(np.float64) @ V[0, 0, 0].astype(np.float64)
    np.testing.assert_allclose(O[0, 0, 0], ref, rtol=1e-14, atol=1e-15)
    prefix = np.cumsum(V[0, 0, 0].astype(np.float64), axis=0) / np.arange(1, S + 1)[:, None]
    np.testing.assert_allclose(O[0, 0, 0], prefix, atol=1e-6)


def test_apply_against_library_matmul_with_indirection(oracle_mod):
    M, L, Hq, Hkv, S, D, B = 5, 3, 4, 2, 21, 10, 4       # S != D, Hq != Hkv
    g = torch.Generator().manual_seed(32)
    maps = torch.softmax(torch.randn(M, L, Hq, S, S, generator=g, dtype=torch.float64), -1).float()
    V = torch.randn(B, 2, Hkv, S, D, generator=g, dtype=torch.float64).float()
    hit = np.array([3, -1, 0, 3], np.int32)
    out = np.full((B, 2, Hq, S, D), -5.0)
    O = oracle_mod.apply(maps.numpy(), hit, V.numpy(), layer_begin=1, out=out)
    for b in range(B):
        if hit[b] < 0:
            assert (O[b] == -5.0).all()                    # misses are not written
            continue
        for l in range(2):
            for h in range(Hq):
                ref = maps[hit[b], 1 + l, h].double() @ V[b, l, h // (Hq // Hkv)].double()
                np.testing.assert_allclose(O[b, l, h], ref.numpy(), rtol=1e-13, atol=1e-14)


def test_apply_sums_every_column(oracle_mod):
    # a dense (non-causal) map must be used in full: mass above the diagonal counts
    S, D = 6, 3
    A = np.zeros((S, S), np.float32); A[:, S - 1] = 1.0   # every row looks at the LAST token only
    V = _rand((1, 1, 1, S, D), 33)
    O = oracle_mod.apply(A.reshape(1, 1, 1, S, S), np.zeros(1, np.int32), V)
    assert np.array_equal(O[0, 0, 0], np.repeat(V[0, 0, 0, S - 1:].astype(np.float64), S, 0))


def test_apply_linearity_and_convexity(oracle_mod):
    S, D = 33, 7
    g = torch.Generator().manual_seed(34)
    maps = torch.softmax(torch.randn(1, 1, 1, S, S, generator=g, dtype=torch.float64), -1).float().numpy()
    V1, V2 = _rand((1, 1, 1, S, D), 35), _rand((1, 1, 1, S, D), 36)
    hit = np.zeros(1, np.int32)
    O1, O2 = oracle_mod.apply(maps, hit, V1), oracle_mod.apply(maps, hit, V2)
    O12 = oracle_mod.apply(maps, hit, V1 * np.float32(2) + V2 * np.float32(0.5))
    Vmix = (V1 * np.float32(2) + V2 * np.float32(0.5)).astype(np.float64)
    exact_mix = 2 * V1.astype(np.float64) + 0.5 * V2.astype(np.float64)
    np.testing.assert_allclose(O12, 2 * O1 + 0.5 * O2 + oracle_mod.apply(maps, hit, (Vmix - exact_mix)),
                               atol=1e-6)
    rs = maps[0, 0, 0].astype(np.float64).sum(-1, keepdims=True)   # rows sum to ~1 (fp32-rounded)
    lo, hi = V1[0, 0, 0].min(0) * rs, V1[0, 0, 0].max(0) * rs
    assert (O1[0, 0, 0] >= np.minimum(lo, hi) - 1e-12).all()
    assert (O1[0, 0, 0] <= np.maximum(lo, hi) + 1e-12).all()


def test_apply_rejects_bad_index(oracle_mod):
    maps = np.zeros((2, 1, 1, 4, 4), np.float32)
    V = np.zeros((1, 1, 1, 4, 2), np.float32)
    with pytest.raises(RuntimeError):
        oracle_mod.apply(maps, np.array([2], np.int32), V)
    with pytest.raises(RuntimeError):
        oracle_mod.apply(maps, np.array([-2], np.int32), V)


# ------------------------------------------------------- reuse of one's own map == exact

@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 1)])
def test_reusing_own_map_reproduces_exact_attention(oracle_mod, hq, hkv):
    B, S, D = 2, 40, 16
    Q, K, V = _rand((B, hq, S, D), 40), _rand((B, hkv, S, D), 41), _rand((B, hkv, S, D), 42)
    O, P = oracle_mod.attention_exact(Q, K, V, return_map=True)
    hit = np.arange(B, dtype=np.int32)
    # entry b = maps of batch item b, one layer
    for kind, tol in ((oracle_mod.ROUND_F32, 2e-6), (oracle_mod.ROUND_BF16, 2e-2)):
        maps = oracle_mod.round_maps(P, kind).reshape(B, 1, hq, S, S)
        O2 = oracle_mod.apply(maps, hit, V.reshape(B, 1, hkv, S, D))
        err = np.abs(O2[:, 0] - O).max()
        assert err < tol, (kind, err)
    # the error with bf16 maps is a real rounding effect, not zero
    assert err > 1e-5


# ------------------------------------------------------------ storage rounding

def test_bf16_rounding_hand_values(oracle_mod):
    u = 2.0 ** -7                                          # bf16 spacing in [1, 2)
    x = np.array([1.0, 1 + u / 2, 1 + 3 * u / 2, 1 + u / 2 + 2.0 ** -40, 1 + u * 0.49,
                  0.0, -1 - u / 2, 3.0e-39, 2.0 ** -133 * 1.5, 0.1], np.float64)
    want = np.array([1.0, 1.0, 1 + 2 * u, 1 + u, 1.0, 0.0, -1.0,
                     round(3.0e-39 / 2.0 ** -133) * 2.0 ** -133, 2.0 ** -132,
                     0.10009765625], np.float64)
    got = oracle_mod.round_maps(x, oracle_mod.ROUND_BF16).astype(np.float64)
    assert np.array_equal(got, want)


def test_bf16_rounding_matches_library_on_fp32_values(oracle_mod):
    g = torch.Generator().manual_seed(43)
    x = torch.cat([torch.rand(20000, generator=g), torch.randn(20000, generator=g) * 1e-3,
                   torch.rand(1000, generator=g) * 1e-38])
    got = oracle_mod.round_maps(x.double().numpy(), oracle_mod.ROUND_BF16)
    assert np.array_equal(got, x.to(torch.bfloat16).float().numpy())
    got32 = oracle_mod.round_maps(x.double().numpy() * (1 + 2.0 ** -30), oracle_mod.ROUND_F32)
    assert np.array_equal(got32, (x.double() * (1 + 2.0 ** -30)).float().numpy())


def test_stored_map_row_sums(oracle_mod):
    B, H, S, D = 1, 4, 128, 16
    Q, K, V = _rand((B, H, S, D), 44), _rand((B, H, S, D), 45), _rand((B, H, S, D), 46)
    _, P = oracle_mod.attention_exact(Q, K, V, return_map=True)
    bf = oracle_mod.round_maps(P, oracle_mod.ROUND_BF16).astype(np.float64)
    f32 = oracle_mod.round_maps(P, oracle_mod.ROUND_F32).astype(np.float64)
    assert np.abs(bf.sum(-1) - 1).max() <= 4e-3
    assert np.abs(f32.sum(-1) - 1).max() <= 1e-6
    iu = np.triu_indices(S, 1)
    assert (bf[..., iu[0], iu[1]] == 0).all()
