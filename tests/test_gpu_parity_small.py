"""GPU parity, small cases: the HIP library (through the C ABI) against the CPU oracle,
element by element, on seeded inputs whose sizes span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ac():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    from paper_2510_25979_amd import binding
    binding.lib()
    return binding


def _gen(seed):
    return torch.Generator(device="cpu").manual_seed(seed)


def _maps(M, L, H, S, dtype, causal, seed):
    logits = torch.randn(M, L, H, S, S, generator=_gen(seed))
    if causal:
        logits.masked_fill_(torch.ones(S, S, dtype=torch.bool).triu_(1), float("-inf"))
    return torch.softmax(logits, -1).to(dtype)


# ------------------------------------------------------------------------- apply

APPLY_CASES = [
    # B, M, L, Hq, Hkv, S, D, causal, layer_begin, Lc, dtype
    (4, 16, 1, 2, 2, 32, 64, True, 0, 1, torch.float32),      # the tiny fp32 workload's shape
    (3, 5, 2, 4, 2, 45, 24, False, 1, 1, torch.float32),      # odd sizes on the vector-ALU path
    (5, 7, 3, 4, 4, 128, 64, True, 0, 3, torch.bfloat16),     # 1B-shaped heads
    (4, 6, 2, 8, 2, 128, 128, True, 1, 1, torch.bfloat16),    # 8B-shaped heads (4 share a V)
    (3, 4, 1, 2, 2, 96, 64, True, 0, 1, torch.bfloat16),      # one ragged block of rows
    (2, 3, 2, 4, 1, 288, 128, True, 0, 2, torch.bfloat16),    # three row blocks, ragged last
    (2, 3, 1, 2, 2, 160, 64, False, 0, 1, torch.bfloat16),    # dense maps
    (2, 3, 1, 4, 2, 32, 128, False, 0, 1, torch.bfloat16),    # a single 32-row block
    (9, 4, 1, 3, 3, 64, 64, True, 0, 1, torch.bfloat16),      # tile count not a multiple of 8
    (2, 2, 1, 2, 1, 416, 64, True, 0, 1, torch.bfloat16),     # four row blocks, ragged, 2 heads per V
    (1, 2, 1, 1, 1, 1024, 128, True, 0, 1, torch.bfloat16),   # the long-sequence shape, one head
    (2, 2, 1, 2, 2, 224, 128, False, 0, 1, torch.bfloat16),   # dense maps, two chunks, ragged
    (2, 3, 1, 2, 2, 320, 64, True, 0, 1, torch.bfloat16),     # paired row blocks: (2, 0) and the middle one alone
    (2, 2, 1, 2, 1, 160, 64, True, 0, 1, torch.bfloat16),     # one pair, ragged second block
    (1, 2, 1, 2, 2, 1024, 64, True, 0, 1, torch.bfloat16),    # four pairs of row blocks
]


def _build(ac, emb, maps, layout, causal, **kw):
    """Database over dense maps, or over their packed form (converted on the GPU)."""
    if layout == "dense":
        return ac.attncache_build_db(emb.cuda(), maps.cuda(), causal=causal, **kw)
    M, L, Hq, S, _ = maps.shape
    packed = torch.empty(M, L, Hq, ac.packed_tile_elems(S, causal), dtype=torch.bfloat16, device="cuda")
    ac.attncache_pack_maps(maps.cuda(), packed, causal=causal)
    return ac.attncache_build_db(emb.cuda(), packed, causal=causal, seq_len=S, **kw)


@pytest.mark.parametrize("layout", ["dense", "packed"])
@pytest.mark.parametrize("case", APPLY_CASES, ids=lambda c: "B%d-M%d-L%d-H%d/%d-S%d-D%d-%s-%d+%d-%s" % (
    c[0], c[1], c[2], c[3], c[4], c[5], c[6], "causal" if c[7] else "dense", c[8], c[9],
    str(c[10]).split(".")[-1]))
def test_apply_matches_oracle(ac, oracle_mod, case, layout):
    B, M, L, Hq, Hkv, S, D, causal, lb, Lc, dt = case
    if layout == "packed" and dt != torch.bfloat16:
        pytest.skip("the packed layout exists for bf16 maps only")
    maps = _maps(M, L, Hq, S, dt, causal, 100 + S + D)
    V = torch.randn(B, Lc, Hkv, S, D, generator=_gen(200 + S)).to(dt)
    hit = torch.randint(0, M, (B,), generator=_gen(300 + B), dtype=torch.int32)
    if B > 2:
        hit[1] = -1                      # a miss: its output rows must stay untouched
    emb = torch.zeros(M, 16, dtype=torch.float32)
    db = _build(ac, emb, maps, layout, causal, n_kv_heads=Hkv, head_dim=D)
    O = torch.full((B, Lc, Hq, S, D), 7.0, dtype=dt, device="cuda")
    ac.attncache_apply(db, hit.cuda(), V.cuda(), O, layer_begin=lb, layer_count=Lc)
    torch.cuda.synchronize()
    ref = oracle_mod.apply(parity.to_np(maps), hit.numpy(), parity.to_np(V), layer_begin=lb,
                           out=np.full((B, Lc, Hq, S, D), 7.0))
    err = parity.max_abs_err(O, ref)
    assert err <= parity.TOL[dt], err
    if B > 2:
        assert (O[1] == 7.0).all()
    db.close()


@pytest.mark.parametrize("layout", ["dense", "packed"])
def test_apply_identity_map_returns_v_bit_exactly(ac, layout):
    S, D = 128, 64
    maps = torch.eye(S).expand(2, 1, 2, S, S).contiguous().to(torch.bfloat16)
    V = torch.randn(3, 1, 2, S, D, generator=_gen(1)).to(torch.bfloat16)
    db = _build(ac, torch.zeros(2, 16), maps, layout, True, n_kv_heads=2, head_dim=D)
    O = torch.zeros(3, 1, 2, S, D, dtype=torch.bfloat16, device="cuda")
    ac.attncache_apply(db, torch.tensor([0, 1, 0], dtype=torch.int32).cuda(), V.cuda(), O)
    assert torch.equal(O.cpu(), V)


def test_apply_out_of_range_hit_is_a_miss_on_device(ac):
    S, D = 32, 64
    maps = _maps(2, 1, 2, S, torch.bfloat16, True, 5)
    db = ac.attncache_build_db(torch.zeros(2, 16).cuda(), maps.cuda(), n_kv_heads=2, head_dim=D)
    V = torch.randn(2, 1, 2, S, D, generator=_gen(2)).to(torch.bfloat16).cuda()
    O = torch.full((2, 1, 2, S, D), 3.0, dtype=torch.bfloat16, device="cuda")
    ac.attncache_apply(db, torch.tensor([2, -5], dtype=torch.int32).cuda(), V, O)
    assert (O == 3.0).all()
    ac.attncache_apply(db, torch.zeros(0, dtype=torch.int32).cuda(), V[:0], O[:0])   # B = 0


# ------------------------------------------------------------------------- exact

EXACT_CASES = [
    # B, Hq, Hkv, S, D, causal, scale, dtype
    (4, 2, 2, 32, 64, True, 0.0, torch.float32),
    (2, 4, 2, 45, 24, False, 0.3, torch.float32),
    (3, 4, 4, 128, 64, True, 0.0, torch.bfloat16),
    (3, 8, 2, 128, 128, True, 0.0, torch.bfloat16),
    (2, 2, 2, 96, 64, True, 0.0, torch.bfloat16),
    (2, 4, 1, 288, 128, True, 0.0, torch.bfloat16),
    (2, 2, 2, 160, 64, False, 0.2, torch.bfloat16),
    (1, 3, 3, 32, 128, False, 0.0, torch.bfloat16),
    (9, 3, 1, 416, 64, True, 0.0, torch.bfloat16),
    (1, 2, 1, 1024, 128, True, 0.0, torch.bfloat16),   # eight row blocks, up to 16 key chunks
    (2, 2, 2, 224, 128, False, 0.0, torch.bfloat16),   # dense, ragged last chunk (32 keys)
    (2, 4, 2, 640, 64, True, 0.15, torch.bfloat16),
]


@pytest.mark.parametrize("case", EXACT_CASES, ids=lambda c: "B%d-H%d/%d-S%d-D%d-%s-%s" % (
    c[0], c[1], c[2], c[3], c[4], "causal" if c[5] else "dense", str(c[7]).split(".")[-1]))
def test_exact_matches_oracle(ac, oracle_mod, case):
    B, Hq, Hkv, S, D, causal, scale, dt = case
    g = _gen(400 + S + D)
    Q = torch.randn(B, Hq, S, D, generator=g).to(dt)
    K = torch.randn(B, Hkv, S, D, generator=g).to(dt)
    V = torch.randn(B, Hkv, S, D, generator=g).to(dt)
    row_sel = None
    if B > 2:
        row_sel = torch.full((B,), -1, dtype=torch.int32)
        row_sel[1] = 4                   # served by the reuse branch: must be skipped
    O = torch.full((B, Hq, S, D), 7.0, dtype=dt, device="cuda")
    ac.attention_exact(Q.cuda(), K.cuda(), V.cuda(), O, causal=causal, scale=scale,
                       row_sel=None if row_sel is None else row_sel.cuda())
    torch.cuda.synchronize()
    ref = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(K), parity.to_np(V), causal=causal,
                                     scale=scale, row_sel=None if row_sel is None else row_sel.numpy(),
                                     out=np.full((B, Hq, S, D), 7.0))
    err = parity.max_abs_err(O, ref)
    assert err <= parity.TOL[dt], err
    if row_sel is not None:
        assert (O[1] == 7.0).all()


PADDED_CASES = [
    # B, Hq, Hkv, S, D, causal, dtype, lengths
    (6, 2, 2, 128, 64, False, torch.bfloat16, [128, 1, 33, 64, 65, 100]),      # encoder-style, resident
    (5, 4, 1, 128, 128, False, torch.bfloat16, [127, 96, 32, 31, 2]),          # four heads share K, V
    (4, 2, 2, 128, 64, True, torch.bfloat16, [128, 70, 5, 64]),                # causal: only the padding rows change
    (3, 2, 2, 96, 128, False, torch.bfloat16, [96, 40, 65]),
    (5, 2, 1, 640, 64, False, torch.bfloat16, [640, 1, 64, 333, 577]),         # streaming: chunks in the padding are skipped
    (4, 2, 2, 416, 128, True, torch.bfloat16, [416, 129, 200, 31]),            # streaming, causal, ragged S
    (1, 1, 1, 1024, 128, False, torch.bfloat16, [700]),
    (4, 3, 1, 45, 24, False, torch.float32, [45, 1, 17, 44]),                  # vector-ALU path
    (3, 2, 2, 32, 64, True, torch.float32, [32, 9, 1]),
]


@pytest.mark.parametrize("case", PADDED_CASES, ids=lambda c: "B%d-H%d/%d-S%d-D%d-%s-%s" % (
    c[0], c[1], c[2], c[3], c[4], "causal" if c[5] else "dense", str(c[6]).split(".")[-1]))
def test_exact_with_sentence_lengths_matches_oracle(ac, oracle_mod, case):
    # a right-padded batch: keys at or beyond the sentence's length are hidden from every row;
    # the padding holds large values that would show in the result if they were read into it
    B, Hq, Hkv, S, D, causal, dt, lens = case
    g = _gen(900 + S + D)
    Q = torch.randn(B, Hq, S, D, generator=g).to(dt)
    K = torch.randn(B, Hkv, S, D, generator=g).to(dt)
    V = torch.randn(B, Hkv, S, D, generator=g).to(dt)
    key_len = torch.tensor(lens, dtype=torch.int32)
    Kc, Vc = K.clone(), V.clone()                    # ordinary values everywhere, for the last part
    for b in range(B):
        K[b, :, lens[b]:] = 3.0
        V[b, :, lens[b]:] = 50.0
    O = torch.full((B, Hq, S, D), 7.0, dtype=dt, device="cuda")
    ac.attention_exact(Q.cuda(), K.cuda(), V.cuda(), O, causal=causal, key_len=key_len.cuda())
    torch.cuda.synchronize()
    ref = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(K), parity.to_np(V), causal=causal,
                                     key_len=key_len.numpy())
    err = parity.max_abs_err(O, ref)
    assert err <= parity.TOL[dt], err
    # lengths outside [1, S] are clamped, and the full length equals the call without lengths
    wild = torch.tensor([S + 9 if b % 2 else 0 for b in range(B)], dtype=torch.int32)
    O2 = torch.empty_like(O)
    ac.attention_exact(Q.cuda(), Kc.cuda(), Vc.cuda(), O2, causal=causal, key_len=wild.cuda())
    torch.cuda.synchronize()
    ref2 = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(Kc), parity.to_np(Vc), causal=causal,
                                      key_len=wild.clamp(1, S).numpy())
    assert parity.max_abs_err(O2, ref2) <= parity.TOL[dt]
    O3 = torch.empty_like(O)
    ac.attention_exact(Q.cuda(), Kc.cuda(), Vc.cuda(), O3, causal=causal)
    torch.cuda.synchronize()
    assert torch.equal(O3[1::2], O2[1::2])


def test_exact_many_tiles_per_workgroup_with_routing(ac, oracle_mod):
    # enough (batch, head) tiles that one workgroup walks several of them back to back, with
    # some batch items routed away (their tiles are skipped in the middle of a walk)
    B, H, S, D = 33, 128, 32, 64
    g = _gen(11)
    Q = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    K = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    V = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    row_sel = torch.full((B,), -1, dtype=torch.int32)
    row_sel[[0, 5, 6, 32]] = 1
    O = torch.full((B, H, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
    ac.attention_exact(Q.cuda(), K.cuda(), V.cuda(), O, row_sel=row_sel.cuda())
    torch.cuda.synchronize()
    ref = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(K), parity.to_np(V),
                                     row_sel=row_sel.numpy(), out=np.full((B, H, S, D), 7.0))
    assert parity.max_abs_err(O, ref) <= 2e-2
    assert (O[[0, 5, 6, 32]] == 7.0).all()


def test_exact_routed_walk_beyond_one_mask_of_candidates(ac, oracle_mod):
    # A routed launch has at most 4,096 workgroups and a workgroup looks at 64 candidate tiles
    # per scan of the routing flags: with more than 262,144 (item, head) tiles a walk needs a
    # second scan.  Sampled tiles against the oracle (the first and last tiles, and tiles on both
    # sides of the second scan), routed-away items untouched.
    B, H, S, D = 2100, 128, 32, 64
    assert B * H > 64 * 4096
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(4711)
    Q = torch.randn(B, H, S, D, generator=g, device=dev).to(torch.bfloat16)
    K = torch.randn(B, H, S, D, generator=g, device=dev).to(torch.bfloat16)
    V = torch.randn(B, H, S, D, generator=g, device=dev).to(torch.bfloat16)
    away = torch.rand(B, generator=g, device=dev) < 0.5
    away[[0, 2047, 2048, B - 1]] = torch.tensor([False, True, False, False], device=dev)
    row_sel = torch.where(away, torch.ones(B, dtype=torch.int32, device=dev),
                          -torch.ones(B, dtype=torch.int32, device=dev))
    O = torch.full((B, H, S, D), 7.0, dtype=torch.bfloat16, device=dev)
    ac.attention_exact(Q, K, V, O, row_sel=row_sel)
    torch.cuda.synchronize()
    assert (O[away] == 7.0).all()
    live = (~away).nonzero().flatten().cpu().tolist()
    rng = np.random.default_rng(5)
    items = sorted({0, 2048, B - 1, live[len(live) // 2], *rng.choice(live, 12).tolist()})
    for b in items:
        heads = sorted({0, H - 1, *rng.integers(0, H, 3).tolist()})
        ref = oracle_mod.attention_exact(parity.to_np(Q[b, heads]).reshape(1, len(heads), S, D),
                                         parity.to_np(K[b, heads]).reshape(1, len(heads), S, D),
                                         parity.to_np(V[b, heads]).reshape(1, len(heads), S, D))
        assert parity.max_abs_err(O[b, heads].contiguous().unsqueeze(0), ref) <= 2e-2, b
    # every tile of a live item was written (nothing kept the fill value in a whole tile)
    untouched = (O[~away] == 7.0).flatten(2).all(-1)
    assert not untouched.any()


def test_exact_large_logits_stay_finite(ac, oracle_mod):
    # peaked softmax: logits of magnitude ~60 must not overflow the online rescaling
    B, H, S, D = 1, 2, 256, 64
    g = _gen(7)
    Q = (torch.randn(B, H, S, D, generator=g) * 6).to(torch.bfloat16)
    K = (torch.randn(B, H, S, D, generator=g) * 6).to(torch.bfloat16)
    V = torch.randn(B, H, S, D, generator=g).to(torch.bfloat16)
    O = torch.empty(B, H, S, D, dtype=torch.bfloat16, device="cuda")
    ac.attention_exact(Q.cuda(), K.cuda(), V.cuda(), O)
    ref = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(K), parity.to_np(V))
    assert parity.max_abs_err(O, ref) <= 2e-2


def test_reusing_own_map_reproduces_exact_attention_on_gpu(ac, oracle_mod):
    # maps computed (by the oracle) from the same Q, K and stored in bf16: the reuse branch
    # must agree with the recompute branch
    B, Hq, Hkv, S, D = 3, 4, 2, 128, 64
    g = _gen(8)
    Q = torch.randn(B, Hq, S, D, generator=g).to(torch.bfloat16)
    K = torch.randn(B, Hkv, S, D, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, S, D, generator=g).to(torch.bfloat16)
    _, P = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(K), parity.to_np(V), return_map=True)
    maps = torch.from_numpy(oracle_mod.round_maps(P, oracle_mod.ROUND_BF16)).to(torch.bfloat16)
    maps = maps.reshape(B, 1, Hq, S, S).contiguous()
    db = _build(ac, torch.zeros(B, 16), maps, "packed", True, n_kv_heads=Hkv, head_dim=D)
    O_reuse = torch.empty(B, 1, Hq, S, D, dtype=torch.bfloat16, device="cuda")
    ac.attncache_apply(db, torch.arange(B, dtype=torch.int32).cuda(), V.reshape(B, 1, Hkv, S, D).cuda(), O_reuse)
    O_exact = torch.empty(B, Hq, S, D, dtype=torch.bfloat16, device="cuda")
    ac.attention_exact(Q.cuda(), K.cuda(), V.cuda(), O_exact)
    assert (O_reuse[:, 0].float() - O_exact.float()).abs().max().item() <= 4e-2
    ref = oracle_mod.attention_exact(parity.to_np(Q), parity.to_np(K), parity.to_np(V))
    assert parity.max_abs_err(O_exact, ref) <= 2e-2
    assert parity.max_abs_err(O_reuse[:, 0].contiguous(), ref) <= 2e-2


# ------------------------------------------------------------------------ search

SEARCH_CASES = [
    # N, E, B, k, dtype, metric, normalise
    (1024, 128, 4, 1, torch.float32, "ip", False),      # the tiny workload
    (1024, 128, 4, 3, torch.float32, "l2", False),
    (777, 40, 5, 4, torch.float32, "ip", False),
    (1000, 256, 64, 1, torch.float16, "ip", True),
    (10000, 256, 64, 1, torch.float16, "ip", True),     # the 1B-shaped workload's index
    (4097, 256, 100, 1, torch.float16, "ip", True),     # ragged rows and queries
    (1024, 512, 16, 4, torch.float16, "ip", True),      # the long-sequence workload's index
    (5000, 128, 300, 1, torch.float16, "ip", True),     # more than one query super-block
    (77, 48, 3, 64, torch.float16, "ip", False),        # k = AC_MAX_K > rows per group
    (3000, 256, 33, 8, torch.float16, "ip", True),
    (600, 40, 7, 2, torch.float16, "ip", False),        # E % 16 != 0: vector-ALU path on fp16
    (900, 64, 6, 2, torch.float16, "l2", False),
    (140000, 64, 40, 4, torch.float16, "ip", True),     # several row passes per workgroup
    (70001, 256, 130, 1, torch.float16, "ip", True),    # large batch: three chunks per workgroup, ragged end
    (66000, 512, 70, 2, torch.float16, "ip", True),     # large batch, widest rows, re-scored top-2
    (50021, 256, 5, 1, torch.float16, "ip", True),      # large database, a handful of queries
    (60000, 128, 33, 3, torch.float16, "ip", True),     # large database, one query past a block
    (50000, 512, 1, 1, torch.float16, "ip", True),      # large database, a single query
    (32768, 128, 9, 5, torch.float16, "ip", True),      # top-k, the most 32-row groups (1,024)
    (40000, 256, 10, 3, torch.float16, "ip", True),     # top-k just above that: one group per workgroup
    (2021, 64, 70, 6, torch.float16, "ip", True),       # top-k, ragged last group, three query blocks
]


def _run_search(ac, emb, q, k, theta, metric, map_of=None):
    M = emb.shape[0] if map_of is None else int(map_of.max()) + 1
    maps = torch.zeros(M, 1, 1, 32, 32, dtype=torch.float32)
    db = ac.attncache_build_db(emb.cuda(), maps.cuda(), n_kv_heads=1, head_dim=8, metric=metric,
                               map_of=None if map_of is None else map_of.cuda())
    B = q.shape[0]
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, k), dtype=torch.uint8, device="cuda")
    idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    score = torch.zeros(B, k, dtype=torch.float32, device="cuda")
    hit = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ac.attncache_search(db, q.cuda(), k, theta, idx, score, hit, ws)
    torch.cuda.synchronize()
    db.close()
    return idx, score, hit


@pytest.mark.parametrize("case", SEARCH_CASES, ids=lambda c: "N%d-E%d-B%d-k%d-%s-%s" % (
    c[0], c[1], c[2], c[3], str(c[4]).split(".")[-1], c[5]))
def test_search_matches_oracle(ac, oracle_mod, case):
    N, E, B, k, dt, metric, normalise = case
    g = _gen(500 + N + E)
    raw = torch.randn(N, E, generator=g)
    emb = (raw / raw.norm(dim=-1, keepdim=True) if normalise else raw).to(dt)
    rows = torch.randint(0, N, (B,), generator=g)
    qf = raw[rows] + 0.1 * torch.randn(B, E, generator=g)
    qf[::3] = torch.randn(qf[::3].shape, generator=g)          # every third query is a miss
    q = (qf / qf.norm(dim=-1, keepdim=True) if normalise else qf).to(dt)
    m = ac.AC_IP if metric == "ip" else ac.AC_L2
    theta = 0.9 if (normalise and metric == "ip") else (0.0 if metric == "ip" else -1.0)
    idx, score, hit = _run_search(ac, emb, q, k, theta, m)
    exempt = parity.check_search(oracle_mod, q, emb, k, theta, m, None, idx, score, hit)
    assert exempt <= max(1, B * k // 50), exempt


def _random_search_shapes(n, seed):
    """Seeded shapes across every search path: sizes around the 32- and 128-row boundaries,
    every feature width class, one to a few query blocks, k from 1 to the limit."""
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        dt = torch.float16 if rng.random() < 0.8 else torch.float32
        metric = "ip" if rng.random() < 0.8 else "l2"
        E = int(rng.choice([16, 32, 40, 48, 64, 96, 128, 256, 512]))
        N = int(rng.choice([1, 2, 31, 32, 33, 127, 128, 129, 255, 257, 1000, 1024, 2047, 4099]))
        N += int(rng.integers(0, 3)) if N > 2 else 0
        B = int(rng.choice([1, 2, 31, 32, 33, 64, 65, 100, 129]))
        k = int(min(N, rng.choice([1, 1, 2, 3, 5, 8, 17, 64])))
        shapes.append((N, E, B, k, dt, metric))
    return shapes


@pytest.mark.parametrize("case", _random_search_shapes(40, 20251128),
                         ids=lambda c: "N%d-E%d-B%d-k%d-%s-%s" % (c[0], c[1], c[2], c[3],
                                                                   str(c[4]).split(".")[-1], c[5]))
def test_search_seeded_random_shapes_match_oracle(ac, oracle_mod, case):
    N, E, B, k, dt, metric = case
    g = _gen(7000 + 13 * N + 7 * E + B + k)
    raw = torch.randn(N, E, generator=g)
    emb = (raw / raw.norm(dim=-1, keepdim=True)).to(dt)
    rows = torch.randint(0, N, (B,), generator=g)
    qf = raw[rows] + 0.2 * torch.randn(B, E, generator=g)
    qf[::4] = torch.randn(qf[::4].shape, generator=g)
    q = (qf / qf.norm(dim=-1, keepdim=True)).to(dt)
    m = ac.AC_IP if metric == "ip" else ac.AC_L2
    theta = 0.8 if metric == "ip" else 0.4
    map_of = torch.randint(0, 9, (N,), generator=g).int()
    idx, score, hit = _run_search(ac, emb, q, k, theta, m, map_of=map_of)
    exempt = parity.check_search(oracle_mod, q, emb, k, theta, m, map_of, idx, score, hit)
    assert exempt <= max(1, B * k // 25), exempt


NAN_CASES = [
    # N, E, B, k, dtype, metric: one per phase-1 kernel and finalising kernel
    (1000, 256, 8, 1, torch.float16, "ip"),      # row-stationary matrix-core kernel, k = 1
    (3000, 256, 8, 4, torch.float16, "ip"),      # the same with the re-scoring top-k
    (50021, 256, 6, 1, torch.float16, "ip"),     # query-stationary kernel, one query block per wave
    (60000, 128, 140, 1, torch.float16, "ip"),   # query-stationary kernel, two query blocks per wave
    (60000, 128, 33, 3, torch.float16, "ip"),    # query-stationary kernel + re-scoring top-k
    (777, 40, 5, 2, torch.float32, "l2"),        # vector-ALU kernel
]


@pytest.mark.parametrize("case", NAN_CASES, ids=lambda c: "N%d-E%d-B%d-k%d-%s-%s" % (
    c[0], c[1], c[2], c[3], str(c[4]).split(".")[-1], c[5]))
def test_search_query_with_nan_is_a_miss_and_the_others_are_unaffected(ac, oracle_mod, case):
    # every score of a query that holds a NaN is NaN, so no row ever ranks: the finalising
    # kernels must report a miss without looking up map_of at the "no row" index
    N, E, B, k, dt, metric = case
    g = _gen(900 + N + E + B)
    raw = torch.randn(N, E, generator=g)
    emb = (raw / raw.norm(dim=-1, keepdim=True)).to(dt)
    rows = torch.randint(0, N, (B,), generator=g)
    q = emb[rows].clone()
    bad = [0, B - 1] if B > 1 else [0]
    for b in bad:
        q[b, (7 * b) % E] = float("nan")
    m = ac.AC_IP if metric == "ip" else ac.AC_L2
    theta = 0.9 if metric == "ip" else 0.5
    map_of = (torch.arange(N) % 16).int()
    idx, score, hit = _run_search(ac, emb, q, k, theta, m, map_of=map_of)
    idx, hit = idx.cpu(), hit.cpu()
    good = [b for b in range(B) if b not in bad]
    for b in bad:
        assert hit[b] == -1
        assert ((idx[b] == -1) | ((idx[b] >= 0) & (idx[b] < N))).all()
    assert (idx[good, 0].long() == rows[good]).all()
    assert (hit[good].long() == map_of[rows[good]].long()).all()


def test_search_large_database_duplicates_give_the_lowest_row(ac, oracle_mod):
    # the query-stationary kernel remembers only the winning 32-row block and the finalising
    # kernel re-scores it: copies of the best row in the same block, in another block of the
    # same group and in another group must all lose to the lowest row
    N, E, B = 66000, 128, 70
    g = _gen(4242)
    raw = torch.randn(N, E, generator=g)
    emb = (raw / raw.norm(dim=-1, keepdim=True)).half()
    rows = 100 + 200 * torch.randperm(100, generator=g)[:B]      # far enough apart not to collide
    for r in rows.tolist():
        emb[r + 3] = emb[r]            # usually the same 32-row block
        emb[r + 64] = emb[r]           # the next chunk of the same group
        emb[r + 40000] = emb[r]        # a different group
    q = emb[rows].clone()
    idx, score, hit = _run_search(ac, emb, q, 1, 0.9, ac.AC_IP)
    assert torch.equal(idx[:, 0].cpu().long(), rows)
    parity.check_search(oracle_mod, q, emb, 1, 0.9, ac.AC_IP, None, idx, score, hit)


def test_search_ties_take_the_lowest_index(ac, oracle_mod):
    g = _gen(9)
    N, E = 2000, 256
    emb = torch.randn(N, E, generator=g)
    emb = (emb / emb.norm(dim=-1, keepdim=True)).to(torch.float16)
    dup = [5, 130, 131, 1029, 1999]                  # identical rows across lanes, waves, groups
    emb[dup] = emb[5].clone()
    q = emb[[5, 700]].clone()
    idx, score, hit = _run_search(ac, emb, q, 5, 0.5, ac.AC_IP)
    assert idx[0].tolist() == dup
    assert len(set(score[0].tolist())) == 1
    idx1, _, hit1 = _run_search(ac, emb, q, 1, 0.5, ac.AC_IP)
    assert idx1[:, 0].tolist() == [5, 700] and hit1.tolist() == [5, 700]


def test_search_map_of_and_threshold(ac, oracle_mod):
    g = _gen(10)
    N, E, M = 3000, 256, 100
    raw = torch.randn(N, E, generator=g)
    emb = (raw / raw.norm(dim=-1, keepdim=True)).to(torch.float16)
    map_of = (torch.arange(N) % M).to(torch.int32)
    rows = torch.tensor([2999, 100, 250, 7])
    qf = raw[rows] + 0.1 * torch.randn(4, E, generator=g)
    qf[3] = torch.randn(E, generator=g)
    q = (qf / qf.norm(dim=-1, keepdim=True)).to(torch.float16)
    idx, score, hit = _run_search(ac, emb, q, 1, 0.9, ac.AC_IP, map_of=map_of)
    assert idx[:3, 0].tolist() == rows[:3].tolist()
    assert hit.tolist() == [2999 % M, 0, 250 % M, -1]
    parity.check_search(oracle_mod, q, emb, 1, 0.9, ac.AC_IP, map_of, idx, score, hit)


# ------------------------------------------------------------------ error paths

def test_whole_step_replayed_from_a_hip_graph_matches_eager(ac, oracle_mod):
    # search -> reuse -> exact on the misses, captured once into a HIP graph and replayed with
    # new inputs written into the same buffers; every replay must equal the eager result, with
    # eager work and synchronisations of the program's own between the replays
    B, M, L, Hq, Hkv, S, D, E = 8, 64, 2, 4, 2, 128, 64, 64
    g = _gen(77)
    maps = _maps(M, L, Hq, S, torch.bfloat16, True, 78)
    emb = torch.nn.functional.normalize(torch.randn(M, E, generator=g), dim=-1).half()
    db = _build(ac, emb, maps, "packed", True, n_kv_heads=Hkv, head_dim=D)
    dev = torch.device("cuda")
    q = torch.empty(B, E, dtype=torch.float16, device=dev)
    Q = torch.empty(B, L * Hq, S, D, dtype=torch.bfloat16, device=dev)
    K = torch.empty(B, L * Hkv, S, D, dtype=torch.bfloat16, device=dev)
    V = torch.empty(B, L * Hkv, S, D, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, 1), dtype=torch.uint8, device=dev)
    idx = torch.empty(B, 1, dtype=torch.int32, device=dev)
    score = torch.empty(B, 1, dtype=torch.float32, device=dev)
    hit = torch.empty(B, dtype=torch.int32, device=dev)
    O = torch.empty(B, L * Hq, S, D, dtype=torch.bfloat16, device=dev)

    def step(out):
        ac.attncache_search(db, q, 1, 0.8, idx, score, hit, ws)
        ac.attncache_apply(db, hit, V.view(B, L, Hkv, S, D), out.view(B, L, Hq, S, D))
        ac.attention_exact(Q, K, V, out, causal=True, row_sel=hit)

    def new_inputs(seed):
        gg = _gen(seed)
        rows = torch.randint(0, M, (B,), generator=gg)
        qq = emb[rows].float() + 0.02 * torch.randn(B, E, generator=gg)
        qq[::3] = torch.randn(B, E, generator=gg)[::3]            # every third query misses
        q.copy_(torch.nn.functional.normalize(qq, dim=-1).half())
        for t in (Q, K, V):
            t.copy_(torch.randn(t.shape, generator=gg).to(torch.bfloat16))

    new_inputs(1)
    step(O)                                                       # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(O)
    torch.cuda.synchronize()
    for seed in (2, 3, 4):
        new_inputs(seed)
        O.fill_(5.0)
        graph.replay()
        torch.cuda.synchronize()
        got, got_hit = O.clone(), hit.clone()
        eager = torch.full_like(O, 5.0)
        step(eager)
        torch.cuda.synchronize()
        assert torch.equal(got_hit, hit)
        assert (hit >= 0).any() and (hit < 0).any()
        assert torch.equal(got, eager), seed
    db.close()


@pytest.mark.parametrize("causal", [True, False])
def test_pack_maps_writes_the_documented_layout(ac, causal):
    # the library's packer against the test suite's own reading of the documented layout
    M, L, Hq, S = 2, 1, 3, 160
    maps = _maps(M, L, Hq, S, torch.bfloat16, causal, 880)
    packed = torch.empty(M, L, Hq, ac.packed_tile_elems(S, causal), dtype=torch.bfloat16, device="cuda")
    ac.attncache_pack_maps(maps.cuda(), packed, causal=causal)
    torch.cuda.synchronize()
    ph, dh = parity.to_np(packed), parity.to_np(maps)
    for m in range(M):
        for h in range(Hq):
            assert np.array_equal(parity.unpack_map(ph[m, 0, h], S, causal), dh[m, 0, h])


def test_per_layer_search_and_reuse_chain_from_one_graph(ac, oracle_mod):
    # per-layer mode (every layer searches its own feature store and reuses or recomputes on
    # its own): L handles over ONE map store, each with its own feature vectors, driven with
    # layer_begin = l; the whole chain of L x (search, reuse, exact) launches is one HIP graph
    B, M, L, Hq, Hkv, S, D, E = 6, 32, 3, 4, 2, 128, 64, 32
    g = _gen(1200)
    maps = _maps(M, L, Hq, S, torch.bfloat16, True, 1201)
    packed = torch.empty(M, L, Hq, ac.packed_tile_elems(S, True), dtype=torch.bfloat16, device="cuda")
    ac.attncache_pack_maps(maps.cuda(), packed, causal=True)
    embs = [torch.nn.functional.normalize(torch.randn(M, E, generator=g), dim=-1).half() for _ in range(L)]
    dbs = [ac.attncache_build_db(embs[l].cuda(), packed, n_kv_heads=Hkv, head_dim=D, causal=True, seq_len=S)
           for l in range(L)]
    dev = torch.device("cuda")
    q = [torch.empty(B, E, dtype=torch.float16, device=dev) for _ in range(L)]
    Q = torch.empty(L, B, 1, Hq, S, D, dtype=torch.bfloat16, device=dev)
    K = torch.empty(L, B, 1, Hkv, S, D, dtype=torch.bfloat16, device=dev)
    V = torch.empty(L, B, 1, Hkv, S, D, dtype=torch.bfloat16, device=dev)
    O = torch.empty(L, B, 1, Hq, S, D, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(ac.attncache_workspace_bytes(dbs[0].desc, B, 1), dtype=torch.uint8, device=dev)
    idx = torch.empty(L, B, 1, dtype=torch.int32, device=dev)
    score = torch.empty(L, B, 1, dtype=torch.float32, device=dev)
    hit = torch.empty(L, B, dtype=torch.int32, device=dev)

    def chain(out):
        for l in range(L):
            ac.attncache_search(dbs[l], q[l], 1, 0.8, idx[l], score[l], hit[l], ws)
            ac.attncache_apply(dbs[l], hit[l], V[l], out[l], layer_begin=l, layer_count=1)
            ac.attention_exact(Q[l].view(B, Hq, S, D), K[l].view(B, Hkv, S, D), V[l].view(B, Hkv, S, D),
                               out[l].view(B, Hq, S, D), causal=True, row_sel=hit[l])

    def new_inputs(seed):
        gg = _gen(seed)
        want = torch.full((L, B), -1, dtype=torch.int64)
        for l in range(L):
            rows = torch.randint(0, M, (B,), generator=gg)
            qq = embs[l][rows].float() + 0.02 * torch.randn(B, E, generator=gg)
            miss = torch.rand(B, generator=gg) < 0.4            # a different hit pattern per layer
            qq[miss] = torch.randn(B, E, generator=gg)[miss]
            q[l].copy_(torch.nn.functional.normalize(qq, dim=-1).half())
            want[l] = torch.where(miss, torch.full_like(rows, -1), rows)
        for t in (Q, K, V):
            t.copy_(torch.randn(t.shape, generator=gg).to(torch.bfloat16))
        return want

    new_inputs(1)
    chain(O)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            chain(O)
    torch.cuda.synchronize()
    maps_np = parity.to_np(maps)
    for seed in (2, 3):
        want = new_inputs(seed)
        O.fill_(5.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(hit.cpu().long(), want)
        for l in range(L):
            h = hit[l].cpu().numpy()
            ref = oracle_mod.attention_exact(parity.to_np(Q[l, :, 0]), parity.to_np(K[l, :, 0]),
                                             parity.to_np(V[l, :, 0]), causal=True, row_sel=h,
                                             out=np.full((B, Hq, S, D), 5.0))
            ref = oracle_mod.apply(maps_np[:, l:l + 1], h, parity.to_np(V[l]),
                                   out=ref.reshape(B, 1, Hq, S, D))
            assert parity.max_abs_err(O[l], ref) <= 2e-2, (seed, l)
    for db in dbs:
        db.close()


INSERT_CASES = [
    # B, L, Hq, Hkv, S, D, causal
    (3, 2, 4, 2, 128, 64, True),
    (2, 1, 2, 2, 96, 128, True),
    (2, 1, 2, 1, 288, 64, True),      # three key chunks, ragged last row block
    (2, 1, 2, 2, 160, 128, False),    # dense maps, ragged last chunk
    (2, 1, 2, 1, 512, 128, True),     # four row blocks, up to eight 64-key chunks, shared K and V
    (2, 2, 2, 2, 352, 64, False),     # dense maps, 32 keys in the last chunk, one wave in the last row block
    (2, 1, 2, 2, 32, 64, True),       # a single 32-row block: one active wave, half a chunk of keys
    (2, 1, 4, 1, 32, 128, False),     # the same, four heads on one K and V
    (2, 1, 2, 2, 64, 128, True),      # exactly one chunk
]


@pytest.mark.parametrize("padded", [False, True], ids=["full", "padded"])
@pytest.mark.parametrize("layout", ["dense", "packed"])
@pytest.mark.parametrize("case", INSERT_CASES, ids=lambda c: "B%d-L%d-H%d/%d-S%d-D%d-%s" % (
    c[0], c[1], c[2], c[3], c[4], c[5], "causal" if c[6] else "dense"))
def test_insert_stores_the_oracles_map_and_output(ac, oracle_mod, case, layout, padded):
    B, L, Hq, Hkv, S, D, causal = case
    M, E = 6, 32
    g = _gen(900 + S + D)
    Q = torch.randn(B, L, Hq, S, D, generator=g).to(torch.bfloat16)
    K = torch.randn(B, L, Hkv, S, D, generator=g).to(torch.bfloat16)
    V = torch.randn(B, L, Hkv, S, D, generator=g).to(torch.bfloat16)
    feat = torch.randn(B, E, generator=g).half()
    key_len = None
    if padded:       # a right-padded batch: the stored map must hold exact zeros in the padding
        key_len = torch.tensor([max(1, S - 27), min(33, S), S][:B], dtype=torch.int32)
        for b in range(B):
            K[b, :, :, key_len[b]:] = 3.0
            V[b, :, :, key_len[b]:] = 50.0
    tile = ac.packed_tile_elems(S, causal) if layout == "packed" else S * S
    sentinel = 0.5
    maps = torch.full((M, L, Hq, tile), sentinel, dtype=torch.bfloat16, device="cuda")
    emb = torch.zeros(M, E, dtype=torch.float16, device="cuda")
    db = ac.attncache_build_db(emb, maps if layout == "packed" else maps.view(M, L, Hq, S, S),
                               n_kv_heads=Hkv, head_dim=D, causal=causal, seq_len=S)
    slot = torch.tensor(([4, -1, 1] if B == 3 else [3, 0]), dtype=torch.int32)
    O = torch.full((B, L, Hq, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
    ac.attncache_insert(db, Q.cuda(), K.cuda(), V.cuda(), O, slot=slot.cuda(), feat=feat.cuda(),
                        key_len=None if key_len is None else key_len.cuda())
    torch.cuda.synchronize()

    maps_h = parity.to_np(maps)
    for l in range(L):
        ref_O, P = oracle_mod.attention_exact(parity.to_np(Q[:, l]), parity.to_np(K[:, l]),
                                              parity.to_np(V[:, l]), causal=causal, return_map=True,
                                              key_len=None if key_len is None else key_len.numpy())
        assert parity.max_abs_err(O[:, l].contiguous(), ref_O) <= 2e-2
        P_r = oracle_mod.round_maps(P, oracle_mod.ROUND_BF16)
        for b in range(B):
            if slot[b] < 0:
                continue
            for h in range(Hq):
                stored = maps_h[slot[b], l, h]
                got = parity.unpack_map(stored, S, causal) if layout == "packed" else stored.reshape(S, S)
                parity.check_stored_map(got, P_r[b, h])
    # nothing else was touched
    used = {int(x) for x in slot if x >= 0}
    for m in range(M):
        if m not in used:
            assert (maps_h[m] == sentinel).all()
            assert (emb[m] == 0).all()
    for b in range(B):
        if slot[b] >= 0:
            assert torch.equal(emb[int(slot[b])].cpu(), feat[b])
    db.close()


def _random_attention_shapes(n, seed):
    """Seeded shapes across the bf16 kernels' variants: resident and streaming lengths (ragged
    row blocks and key chunks), both head widths, head groupings, layouts, padded batches."""
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        S = int(rng.choice([32, 64, 96, 128, 160, 192, 256, 288, 352, 448]))
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 3]))
        grp = int(rng.choice([1, 2, 4]))
        L = int(rng.choice([1, 2]))
        B = int(rng.choice([1, 2, 3]))
        shapes.append((B, L, Hkv * grp, Hkv, S, D, bool(rng.random() < 0.6),
                       "packed" if rng.random() < 0.6 else "dense", bool(rng.random() < 0.4)))
    return shapes


@pytest.mark.parametrize("case", _random_attention_shapes(24, 20251129),
                         ids=lambda c: "B%d-L%d-H%d/%d-S%d-D%d-%s-%s-%s" % (
                             c[0], c[1], c[2], c[3], c[4], c[5], "causal" if c[6] else "dense", c[7],
                             "padded" if c[8] else "full"))
def test_exact_insert_and_reuse_on_seeded_random_shapes(ac, oracle_mod, case):
    # one chain per shape: exact attention, the same computed and remembered, and the reuse
    # branch on the remembered maps, each against the oracle
    B, L, Hq, Hkv, S, D, causal, layout, padded = case
    M, E = B + 2, 32
    g = _gen(1300 + 17 * S + D + 5 * Hq + B)
    Q = torch.randn(B, L, Hq, S, D, generator=g).to(torch.bfloat16)
    K = torch.randn(B, L, Hkv, S, D, generator=g).to(torch.bfloat16)
    V = torch.randn(B, L, Hkv, S, D, generator=g).to(torch.bfloat16)
    key_len = None
    if padded:
        key_len = torch.randint(1, S + 1, (B,), generator=g).int()
        key_len[0] = S - 27 if S > 32 else S
    kl = None if key_len is None else key_len.numpy()
    ref, maps_ref = [], []
    for l in range(L):
        o, P = oracle_mod.attention_exact(parity.to_np(Q[:, l]), parity.to_np(K[:, l]), parity.to_np(V[:, l]),
                                          causal=causal, return_map=True, key_len=kl)
        ref.append(o)
        maps_ref.append(oracle_mod.round_maps(P, oracle_mod.ROUND_BF16))

    # exact attention (layers fold into heads)
    O = torch.full((B, L * Hq, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
    ac.attention_exact(Q.view(B, L * Hq, S, D).cuda(), K.view(B, L * Hkv, S, D).cuda(),
                       V.view(B, L * Hkv, S, D).cuda(), O, causal=causal,
                       key_len=None if key_len is None else key_len.cuda())
    torch.cuda.synchronize()
    for l in range(L):
        assert parity.max_abs_err(O[:, l * Hq:(l + 1) * Hq].contiguous(), ref[l]) <= 2e-2

    # computed and remembered
    tile = ac.packed_tile_elems(S, causal) if layout == "packed" else S * S
    maps = torch.zeros(M, L, Hq, tile, dtype=torch.bfloat16, device="cuda")
    emb = torch.zeros(M, E, dtype=torch.float16, device="cuda")
    db = ac.attncache_build_db(emb, maps if layout == "packed" else maps.view(M, L, Hq, S, S),
                               n_kv_heads=Hkv, head_dim=D, causal=causal, seq_len=S)
    slot = torch.randperm(M, generator=g)[:B].int()
    feat = torch.randn(B, E, generator=g).half()
    O2 = torch.full((B, L, Hq, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
    ac.attncache_insert(db, Q.cuda(), K.cuda(), V.cuda(), O2, slot=slot.cuda(), feat=feat.cuda(),
                        key_len=None if key_len is None else key_len.cuda())
    torch.cuda.synchronize()
    maps_h = parity.to_np(maps)
    for l in range(L):
        assert parity.max_abs_err(O2[:, l].contiguous(), ref[l]) <= 2e-2
        for b in range(B):
            for h in range(Hq):
                stored = maps_h[int(slot[b]), l, h]
                got = parity.unpack_map(stored, S, causal) if layout == "packed" else stored.reshape(S, S)
                parity.check_stored_map(got, maps_ref[l][b, h])

    # the reuse branch on what was remembered
    O3 = torch.full((B, L, Hq, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
    ac.attncache_apply(db, slot.cuda(), V.cuda(), O3)
    torch.cuda.synchronize()
    for l in range(L):
        assert parity.max_abs_err(O3[:, l].contiguous(), ref[l]) <= 2e-2
    db.close()


def test_insert_then_search_and_reuse_closes_the_loop(ac, oracle_mod):
    # miss -> compute and remember -> the same input hits and the reuse branch returns the
    # output the recompute branch produced (same rounded map, summed in another order)
    B, M, L, Hq, Hkv, S, D, E = 4, 16, 2, 4, 2, 128, 64, 64
    g = _gen(950)
    Q = torch.randn(B, L, Hq, S, D, generator=g).to(torch.bfloat16).cuda()
    K = torch.randn(B, L, Hkv, S, D, generator=g).to(torch.bfloat16).cuda()
    V = torch.randn(B, L, Hkv, S, D, generator=g).to(torch.bfloat16).cuda()
    feat = torch.nn.functional.normalize(torch.randn(B, E, generator=g), dim=-1).half().cuda()
    maps = torch.zeros(M, L, Hq, ac.packed_tile_elems(S, True), dtype=torch.bfloat16, device="cuda")
    emb = torch.zeros(M, E, dtype=torch.float16, device="cuda")
    db = ac.attncache_build_db(emb, maps, n_kv_heads=Hkv, head_dim=D, causal=True, seq_len=S)
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, 1), dtype=torch.uint8, device="cuda")
    idx = torch.empty(B, 1, dtype=torch.int32, device="cuda")
    score = torch.empty(B, 1, dtype=torch.float32, device="cuda")
    hit = torch.empty(B, dtype=torch.int32, device="cuda")
    ac.attncache_search(db, feat, 1, 0.9, idx, score, hit, ws)
    assert (hit.cpu() == -1).all()                                   # empty database: all miss
    slot = torch.tensor([9, 2, 15, 0], dtype=torch.int32).cuda()
    O_first = torch.empty(B, L, Hq, S, D, dtype=torch.bfloat16, device="cuda")
    # layer by layer, as a model forward would deliver the maps; the feature goes in once
    for l in range(L):
        O_l = torch.empty(B, 1, Hq, S, D, dtype=torch.bfloat16, device="cuda")
        ac.attncache_insert(db, Q[:, l:l + 1].contiguous(), K[:, l:l + 1].contiguous(),
                            V[:, l:l + 1].contiguous(), O_l, slot=slot,
                            feat=feat if l == 0 else None, row_sel=hit, layer_begin=l)
        O_first[:, l:l + 1] = O_l
    ac.attncache_search(db, feat, 1, 0.9, idx, score, hit, ws)
    torch.cuda.synchronize()
    assert torch.equal(hit, slot)
    O_reuse = torch.empty_like(O_first)
    ac.attncache_apply(db, hit, V, O_reuse)
    torch.cuda.synchronize()
    diff = (O_reuse.float() - O_first.float()).abs()
    assert diff.max().item() <= 2e-2
    assert (diff > 0).float().mean().item() <= 0.05                  # mostly bit-equal
    ref = oracle_mod.attention_exact(parity.to_np(Q.view(B, L * Hq, S, D)),
                                     parity.to_np(K.view(B, L * Hkv, S, D)),
                                     parity.to_np(V.view(B, L * Hkv, S, D)))
    assert parity.max_abs_err(O_reuse.view(B, L * Hq, S, D), ref) <= 2e-2
    db.close()


def test_host_resident_maps_are_cached_across_batches(ac, oracle_mod):
    # maps in pinned host memory, a cache of 4 entries in device memory: popular entries are
    # copied once and reused by later batches, eviction takes the least recently used slot,
    # and every batch still equals the oracle
    M, L, Hq, Hkv, S, D = 12, 2, 2, 1, 128, 64
    maps = _maps(M, L, Hq, S, torch.bfloat16, True, 990)
    host_maps = torch.empty(maps.shape, dtype=torch.bfloat16, pin_memory=True)
    host_maps.copy_(maps)
    entry_bytes = L * Hq * S * S * 2
    staging = torch.empty(4 * entry_bytes, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    db = ac.attncache_build_db(torch.zeros(M, 16, device="cuda"), host_maps, n_kv_heads=Hkv,
                               head_dim=D, staging=staging, side_stream=side)
    maps_np = parity.to_np(maps)
    batches = [([3, 3, 7, 1], 3),          # 3 distinct entries: 3 copies
               ([7, 1, 1, 9], 1),          # 7 and 1 are still there: 1 copy
               ([-1, 9, 9, 3], 0),         # a miss, and two cached entries: no copy
               ([0, 2, 4, 5], 4),          # four new entries replace everything
               ([9, 5, 4, 11], 2)]         # 5 and 4 survive, 9 was evicted
    lookups = copies = 0
    for n, (hits, new_copies) in enumerate(batches):
        B = len(hits)
        V = torch.randn(B, L, Hkv, S, D, generator=_gen(1000 + n)).to(torch.bfloat16)
        O = torch.full((B, L, Hq, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
        hit = torch.tensor(hits, dtype=torch.int32)
        ac.attncache_apply(db, hit, V.cuda(), O)
        torch.cuda.synchronize()
        ref = oracle_mod.apply(maps_np, hit.numpy(), parity.to_np(V), out=np.full((B, L, Hq, S, D), 7.0))
        assert parity.max_abs_err(O, ref) <= 2e-2, n
        lookups += len({h for h in hits if h >= 0})
        copies += new_copies
        assert ac.attncache_cache_stats(db) == (lookups, copies), n
    # a layer sub-range is staged without being remembered
    V = torch.randn(1, 1, Hkv, S, D, generator=_gen(1100)).to(torch.bfloat16)
    O = torch.empty(1, 1, Hq, S, D, dtype=torch.bfloat16, device="cuda")
    ac.attncache_apply(db, torch.tensor([5], dtype=torch.int32), V.cuda(), O, layer_begin=1, layer_count=1)
    torch.cuda.synchronize()
    ref = oracle_mod.apply(maps_np[:, 1:2], np.array([5], np.int32), parity.to_np(V))
    assert parity.max_abs_err(O, ref) <= 2e-2
    assert ac.attncache_cache_stats(db) == (lookups + 1, copies + 1)
    ac.attncache_cache_reset(db)
    assert ac.attncache_cache_stats(db) == (0, 0)
    db.close()


def test_empty_batches_and_all_miss_batches_touch_nothing(ac):
    M, L, Hq, Hkv, S, D, E = 4, 1, 2, 2, 32, 64, 32
    emb = torch.randn(M, E).half().cuda()
    maps = torch.zeros(M, L, Hq, S, S, dtype=torch.bfloat16, device="cuda")
    db = ac.attncache_build_db(emb, maps, n_kv_heads=Hkv, head_dim=D)
    ws = torch.empty(max(256, ac.attncache_workspace_bytes(db.desc, 1, 1)), dtype=torch.uint8, device="cuda")
    z = lambda *shape, dt=torch.bfloat16: torch.zeros(*shape, dtype=dt, device="cuda")
    # B = 0 through every entry point
    ac.attncache_search(db, z(0, E, dt=torch.float16), 1, 0.5, z(0, 1, dt=torch.int32),
                        z(0, 1, dt=torch.float32), z(0, dt=torch.int32), ws)
    ac.attncache_apply(db, z(0, dt=torch.int32), z(0, L, Hkv, S, D), z(0, L, Hq, S, D))
    ac.attention_exact(z(0, Hq, S, D), z(0, Hkv, S, D), z(0, Hkv, S, D), z(0, Hq, S, D))
    ac.attncache_insert(db, z(0, L, Hq, S, D), z(0, L, Hkv, S, D), z(0, L, Hkv, S, D), z(0, L, Hq, S, D),
                        slot=z(0, dt=torch.int32))
    # a batch of misses only: the reuse branch writes nothing; a batch of hits only: neither does
    # the recompute branch
    B = 3
    V = torch.randn(B, L, Hkv, S, D, device="cuda").to(torch.bfloat16)
    O = torch.full((B, L, Hq, S, D), 7.0, dtype=torch.bfloat16, device="cuda")
    ac.attncache_apply(db, torch.full((B,), -1, dtype=torch.int32, device="cuda"), V, O)
    ac.attention_exact(V.view(B, Hq, S, D), V.view(B, Hkv, S, D), V.view(B, Hkv, S, D), O.view(B, Hq, S, D),
                       row_sel=torch.zeros(B, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert (O == 7.0).all()
    assert torch.count_nonzero(maps) == 0
    db.close()


def test_error_codes(ac):
    emb = torch.zeros(64, 128, dtype=torch.float16, device="cuda")
    maps = torch.zeros(64, 1, 2, 32, 32, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ac.AttnCacheError) as e:       # maps promised on the device but on the host
        d = ac.DbDesc(n_emb=64, emb_dim=128, emb_dtype=ac.AC_F16, metric=0, n_entries=64, n_layers=1,
                      n_q_heads=2, n_kv_heads=2, head_dim=64, seq_len=32, map_dtype=ac.AC_BF16,
                      causal=1, maps_on_host=0)
        import ctypes
        host = torch.zeros(64 * 2 * 32 * 32, dtype=torch.bfloat16)
        h = ctypes.c_void_p()
        ac._check(ac.lib().attncache_build_db(ctypes.byref(d), emb.data_ptr(), None, host.data_ptr(),
                                              None, 0, None, ctypes.byref(h)), "attncache_build_db")
    assert e.value.status == -9
    db = ac.attncache_build_db(emb, maps, n_kv_heads=2, head_dim=64)
    q = torch.zeros(4, 128, dtype=torch.float16, device="cuda")
    idx = torch.zeros(4, 1, dtype=torch.int32, device="cuda")
    score = torch.zeros(4, 1, device="cuda")
    hit = torch.zeros(4, dtype=torch.int32, device="cuda")
    tiny = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(ac.AttnCacheError) as e:
        ac.attncache_search(db, q, 1, 0.5, idx, score, hit, tiny)
    assert e.value.status == -6
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(ac.AttnCacheError) as e:
        ac.attncache_search(db, q, 65, 0.5, torch.zeros(4, 65, dtype=torch.int32, device="cuda"),
                            torch.zeros(4, 65, device="cuda"), hit, ws)
    assert e.value.status == -5
    with pytest.raises(ac.AttnCacheError) as e:       # misaligned workspace
        ac.attncache_search(db, q, 1, 0.5, idx, score, hit, ws[1:])
    assert e.value.status == -4
    V = torch.zeros(4, 1, 2, 32, 64, dtype=torch.bfloat16, device="cuda")
    O = torch.zeros(4, 1, 2, 32, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ac.AttnCacheError) as e:       # layer range outside the database
        ac.attncache_apply(db, hit, V, O, layer_begin=1, layer_count=1)
    assert e.value.status == -2
    with pytest.raises(ac.AttnCacheError) as e:       # S not a multiple of 32 on the bf16 path
        x = torch.zeros(1, 1, 40, 64, dtype=torch.bfloat16, device="cuda")
        ac.attention_exact(x, x, x, x.clone())
    assert e.value.status == -2
    Qi = torch.zeros(4, 1, 2, 32, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ac.AttnCacheError) as e:       # insertion beyond the database's layers
        ac.attncache_insert(db, Qi, V, V, O, slot=hit, layer_begin=1)
    assert e.value.status == -2
    many = torch.zeros(128, 128, dtype=torch.float16, device="cuda")   # two feature rows per entry
    db2 = ac.attncache_build_db(many, maps, n_kv_heads=2, head_dim=64,
                                map_of=(torch.arange(128, device="cuda") % 64).int())
    with pytest.raises(ac.AttnCacheError) as e:       # a slot must name one feature row
        ac.attncache_insert(db2, Qi, V, V, O, slot=hit, feat=q)
    assert e.value.status == -2
    db2.close()
    f32db = ac.attncache_build_db(torch.zeros(8, 16, device="cuda"),
                                  torch.zeros(8, 1, 2, 32, 32, device="cuda"), n_kv_heads=2, head_dim=64)
    with pytest.raises(ac.AttnCacheError) as e:       # maps are written as bf16 only
        ac.attncache_insert(f32db, Qi, V, V, O, slot=hit)
    assert e.value.status == -3
    f32db.close()
    ac.attncache_search(db, q, 1, 0.5, idx, score, hit, ws)   # the handle still works
    torch.cuda.synchronize()


def test_host_pointers_are_refused_before_any_launch(ac):
    """Raw C-ABI calls (no binding in between) with a pointer in the wrong memory space return
    AC_ERR_MEMSPACE from the library's host-side check: nothing is launched, so every output
    keeps its fill value.  Ordinary and pinned host memory are both refused where device memory
    is required, and a device `hit` is refused where the host reads it."""
    import ctypes
    L_ = ac.lib()
    cf = ctypes.c_float
    M, L, Hq, Hkv, S, D, E, B = 6, 1, 2, 2, 32, 64, 128, 4
    emb = torch.randn(M, E, device="cuda").half()
    maps = torch.zeros(M, L, Hq, S, S, dtype=torch.bfloat16, device="cuda")
    db = ac.attncache_build_db(emb, maps, n_kv_heads=Hkv, head_dim=D)
    dev = lambda *s, dt=torch.bfloat16, fill=7: torch.full(s, fill, dtype=dt, device="cuda")
    host = lambda *s, dt=torch.bfloat16: torch.zeros(*s, dtype=dt)
    pinned = lambda *s, dt=torch.bfloat16: torch.zeros(*s, dtype=dt, pin_memory=True)
    q, idx, score, hit = dev(B, E, dt=torch.float16, fill=0), dev(B, 1, dt=torch.int32), \
        dev(B, 1, dt=torch.float32), dev(B, dt=torch.int32, fill=0)
    ws = dev(1 << 16, dt=torch.uint8)
    V, O, Q = dev(B, L, Hkv, S, D, fill=1), dev(B, L, Hq, S, D), dev(B, L, Hq, S, D, fill=1)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    for bad in (host, pinned):
        hq, hidx, hV, hO, hws = bad(B, E, dt=torch.float16), bad(B, 1, dt=torch.int32), \
            bad(B, L, Hkv, S, D), bad(B, L, Hq, S, D), bad(1 << 16, dt=torch.uint8)
        assert L_.attncache_search(db.handle, p(hq), B, 1, cf(0.5), p(idx), p(score), p(hit), p(ws), 1 << 16, None) == -9
        assert L_.attncache_search(db.handle, p(q), B, 1, cf(0.5), p(hidx), p(score), p(hit), p(ws), 1 << 16, None) == -9
        assert L_.attncache_search(db.handle, p(q), B, 1, cf(0.5), p(idx), p(score), p(hit), p(hws), 1 << 16, None) == -9
        assert L_.attncache_apply(db.handle, p(hit), p(hV), p(O), B, 0, 1, None) == -9
        assert L_.attncache_apply(db.handle, p(hit), p(V), p(hO), B, 0, 1, None) == -9
        assert L_.attncache_apply(db.handle, p(bad(B, dt=torch.int32)), p(V), p(O), B, 0, 1, None) == -9
        assert L_.attention_exact(p(hO), p(V), p(V), p(O), None, None, B, Hq, Hkv, S, D, ac.AC_BF16, 1, cf(0), None) == -9
        assert L_.attention_exact(p(Q), p(V), p(V), p(O), p(bad(B, dt=torch.int32)), None, B, Hq, Hkv, S, D,
                                  ac.AC_BF16, 1, cf(0), None) == -9
        assert L_.attncache_insert(db.handle, None, p(bad(B, dt=torch.int32)), None, None, p(Q), p(V), p(V), p(O),
                                   B, 0, 1, cf(0), None) == -9
        assert L_.attncache_pack_maps(ctypes.byref(db.desc), p(bad(M, L, Hq, S, S)), M, p(maps), None) == -9
        W = torch.zeros(64, 64, device="cuda")
        pw = dev(ac.attncache_project_workspace_bytes(B, 64, 64, 64), dt=torch.uint8)
        assert L_.attncache_project(p(bad(B, 8, 64)), None, p(W), None, p(W), None, p(dev(B, 64, dt=torch.float16)),
                                    B, 8, 64, 64, 64, ac.AC_BF16, ac.AC_F16, 1, p(pw), pw.numel(), None) == -9
    torch.cuda.synchronize()
    assert (idx == 7).all() and (score == 7).all() and (O == 7).all() and torch.count_nonzero(maps) == 0

    # host-resident maps: `hit` is read by the host, so a device pointer is the wrong one
    hmaps = torch.zeros(M, L, Hq, S, S, dtype=torch.bfloat16, pin_memory=True)
    staging = torch.empty(2 * L * Hq * S * S * 2, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    hdb = ac.attncache_build_db(emb, hmaps, n_kv_heads=Hkv, head_dim=D, staging=staging, side_stream=side)
    assert L_.attncache_apply(hdb.handle, p(hit), p(V), p(O), B, 0, 1, None) == -9
    assert L_.attncache_apply(hdb.handle, p(torch.zeros(B, dtype=torch.int32)), p(V), p(O), B, 0, 1, None) == 0
    torch.cuda.synchronize()
    hdb.close()

    # the checks can be switched off (and report their previous state); valid calls work either way
    assert ac.attncache_set_pointer_checks(False) is True
    assert L_.attncache_search(db.handle, p(q), B, 1, cf(0.5), p(idx), p(score), p(hit), p(ws), 1 << 16, None) == 0
    assert ac.attncache_set_pointer_checks(True) is False
    assert L_.attncache_search(db.handle, p(q), B, 1, cf(0.5), p(idx), p(score), p(hit), p(ws), 1 << 16, None) == 0
    torch.cuda.synchronize()
    db.close()
