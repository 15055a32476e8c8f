"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py times.

The whole step runs on the GPU at full size (full database resident, full batch, all layers and
heads); the oracle then checks the search of every query and EVERY output tile of both
branches, each reuse tile from the dense map bytes the database was built from (re-drawn with
the same seed, never read back through the packed form).
"""
import numpy as np
import pytest
import torch

from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    from paper_2510_25979_amd import binding, synth, synthdb
    binding.lib()
    return binding, synth, synthdb


def _sample_tiles(hits, L, Hq, n, seed):
    """(b, l, h) samples over the queries in `hits`, always including the corners."""
    rng = np.random.default_rng(seed)
    picks = {(hits[0], 0, 0), (hits[-1], L - 1, Hq - 1)}
    while len(picks) < min(n, len(hits) * L * Hq):
        picks.add((int(rng.choice(hits)), int(rng.integers(L)), int(rng.integers(Hq))))
    return sorted(picks)


def _worst_tile(got, ref, queries):
    """Max-abs error per (query, layer, head) tile; returns (error, (b, l, h)) of the worst."""
    assert got.shape == ref.shape and np.isfinite(got).all()
    err = np.abs(got - ref).max(axis=(3, 4))
    n, l, h = np.unravel_index(int(err.argmax()), err.shape)
    return float(err[n, l, h]), (int(queries[n]), int(l), int(h))


def _check_reuse_tiles(oracle_mod, store, hit_h, V, O, queries, tol, chunk_bytes=1 << 30):
    """EVERY (query, layer, head) tile of the reuse branch for the given queries against the
    oracle, which multiplies the dense maps the database was built from (re-drawn with the same
    seed) with V.  Returns the number of tiles compared."""
    w = store.w
    L, Hq = w.n_layers, w.n_q_heads
    per = max(1, chunk_bytes // (w.entry_elems * 4))
    # queries grouped by the slice of the store their entry was drawn in: one re-draw per slice
    order = sorted(queries, key=lambda b: int(hit_h[b]))
    done = 0
    for c0 in range(0, len(order), per):
        qs = order[c0:c0 + per]
        A = torch.stack([store.dense_entry(int(hit_h[b])) for b in qs])
        ref = oracle_mod.apply(parity.to_np(A), np.arange(len(qs), dtype=np.int32), parity.to_np(V[qs]))
        del A
        err, where = _worst_tile(O[qs].double().cpu().numpy(), ref, qs)
        assert err <= tol, ("reuse tile", where, err)
        done += len(qs) * L * Hq
    return done


def _check_exact_tiles(oracle_mod, w, Q, K, V, O, queries, tol, chunk_bytes=1 << 30):
    """EVERY (query, layer, head) tile of the recompute branch for the given queries."""
    B, L, Hq, Hkv, S, D = w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    per = max(1, chunk_bytes // (L * Hq * S * D * 4))
    done = 0
    for c0 in range(0, len(queries), per):
        qs = list(queries[c0:c0 + per])
        n = len(qs)
        ref = oracle_mod.attention_exact(parity.to_np(Q[qs]).reshape(n, L * Hq, S, D),
                                         parity.to_np(K[qs]).reshape(n, L * Hkv, S, D),
                                         parity.to_np(V[qs]).reshape(n, L * Hkv, S, D), causal=w.causal)
        err, where = _worst_tile(O[qs].double().cpu().numpy(), ref.reshape(n, L, Hq, S, D), qs)
        assert err <= tol, ("exact tile", where, err)
        done += n * L * Hq
    return done


def _run_workload(env, oracle_mod, cfg, *, expect_reuse_tiles, expect_exact_tiles):
    """One whole step at the workload's full size, exactly as bench.py issues it; then the oracle
    checks the search of every query and every output tile of both branches."""
    ac, synth, synthdb = env
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[cfg]
    B, L, Hq, Hkv, S, D = w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    dt = synth.torch_dtype(w.map_dtype)
    emb, raw, map_of = synth.make_embeddings(w, dev)
    q, planted = synth.make_queries(w, raw, dev)
    del raw
    store = synthdb.SynthMapStore(w, dev, layout="packed")
    Q, K, V = synth.make_qkv(w, dev)
    sentinel = 3.0
    O = torch.full((B, L, Hq, S, D), sentinel, dtype=dt, device=dev)
    db = ac.attncache_build_db(emb, store.maps, n_kv_heads=Hkv, head_dim=D, causal=w.causal,
                               map_of=map_of, seq_len=S)
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, w.k), dtype=torch.uint8, device=dev)
    idx = torch.empty(B, w.k, dtype=torch.int32, device=dev)
    score = torch.empty(B, w.k, dtype=torch.float32, device=dev)
    hit = torch.empty(B, dtype=torch.int32, device=dev)

    # ---- the step, exactly as bench.py issues it
    Qf, Kf, Vf = Q.view(B, L * Hq, S, D), K.view(B, L * Hkv, S, D), V.view(B, L * Hkv, S, D)
    ac.attncache_search(db, q, w.k, w.theta, idx, score, hit, ws)
    ac.attncache_apply(db, hit, V, O)
    ac.attention_exact(Qf, Kf, Vf, O.view(B, L * Hq, S, D), causal=w.causal, row_sel=hit)
    torch.cuda.synchronize()

    # ---- search: every query against the oracle
    hit_h = hit.cpu().numpy()
    expect_hit = torch.where(planted >= 0, planted % w.n_entries, planted).numpy().astype(np.int32)
    assert np.array_equal(hit_h, expect_hit), "routing differs from the planted hits"
    exempt = parity.check_search(oracle_mod, q, emb, w.k, w.theta, 0, map_of, idx, score, hit)
    assert exempt <= 2

    hits = [b for b in range(B) if hit_h[b] >= 0]
    misses = [b for b in range(B) if hit_h[b] < 0]
    tol = parity.TOL[dt]
    # ---- reuse branch: every tile of every hit
    assert _check_reuse_tiles(oracle_mod, store, hit_h, V, O, hits, tol) == expect_reuse_tiles
    # ---- recompute branch: every tile of every routed miss; when the workload has no miss the
    # routed launch must not have written anything (checked above: every tile equals the reuse
    # result) and the kernel is checked at full size on all queries separately
    if misses:
        assert _check_exact_tiles(oracle_mod, w, Q, K, V, O, misses, tol) == expect_exact_tiles
    else:
        O.fill_(sentinel)
        ac.attention_exact(Qf, Kf, Vf, O.view(B, L * Hq, S, D), causal=w.causal)
        torch.cuda.synchronize()
        assert _check_exact_tiles(oracle_mod, w, Q, K, V, O, list(range(B)), tol) == expect_exact_tiles
    db.close()


def test_workload_1_tiny_fp32_in_full(env, oracle_mod):
    # small enough for the oracle to check every element
    ac, synth, synthdb = env
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[1]
    B, L, Hq, Hkv, S, D = w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    emb, raw, _ = synth.make_embeddings(w, dev)
    q, planted = synth.make_queries(w, raw, dev)
    store = synthdb.SynthMapStore(w, dev)
    Q, K, V = synth.make_qkv(w, dev)
    for metric in (ac.AC_IP, ac.AC_L2):
        db = ac.attncache_build_db(emb, store.maps, n_kv_heads=Hkv, head_dim=D, metric=metric)
        ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, 1), dtype=torch.uint8, device=dev)
        idx = torch.empty(B, 1, dtype=torch.int32, device=dev)
        score = torch.empty(B, 1, device=dev)
        hit = torch.empty(B, dtype=torch.int32, device=dev)
        theta = 0.0 if metric == ac.AC_IP else -1.0
        ac.attncache_search(db, q, 1, theta, idx, score, hit, ws)
        torch.cuda.synchronize()
        assert hit.cpu().tolist() == planted.tolist()          # planted neighbour under both metrics
        parity.check_search(oracle_mod, q, emb, 1, theta, metric, None, idx, score, hit)
        O = torch.zeros(B, L, Hq, S, D, device=dev)
        ac.attncache_apply(db, hit, V, O)
        torch.cuda.synchronize()
        ref = oracle_mod.apply(parity.to_np(store.maps), hit.cpu().numpy(), parity.to_np(V))
        assert parity.max_abs_err(O, ref) <= 1e-4
        db.close()
    Ox = torch.zeros(B, Hq, S, D, device=dev)
    ac.attention_exact(Q[:, 0].contiguous(), K[:, 0].contiguous(), V[:, 0].contiguous(), Ox)
    ref = oracle_mod.attention_exact(parity.to_np(Q[:, 0]), parity.to_np(K[:, 0]), parity.to_np(V[:, 0]))
    assert parity.max_abs_err(Ox, ref) <= 1e-4


def test_workload_2_llama_1b_shaped_full_size_all_32768_reuse_and_all_32768_exact_tiles(env, oracle_mod):
    _run_workload(env, oracle_mod, 2, expect_reuse_tiles=64 * 16 * 32, expect_exact_tiles=64 * 16 * 32)


def test_workload_3_llama_8b_shaped_full_size_all_65536_hit_and_all_65536_miss_tiles(env, oracle_mod):
    _run_workload(env, oracle_mod, 3, expect_reuse_tiles=64 * 32 * 32, expect_exact_tiles=64 * 32 * 32)


def test_workload_4_long_sequence_top4_full_size_all_512_reuse_and_all_512_exact_tiles(env, oracle_mod):
    _run_workload(env, oracle_mod, 4, expect_reuse_tiles=16 * 32, expect_exact_tiles=16 * 32)


# Pinned host memory the GPU machines grant one process: 64 GiB in total, whatever the size of the
# single allocations (measured with a ladder of hipHostMalloc calls; the machine has 295 GiB of
# RAM).  The over-HBM workload's store is therefore 3,200 packed entries of 20 MiB (62.5 GiB)
# instead of 12,800; entry size, index size, batch and popularity law are the workload's.
HOST_ENTRY_LADDER = (3200, 2400, 1600, 800)


def _lru_copies(batches_of_entries, n_slots):
    """Copies the documented policy must issue: per call the distinct entries that are cached at
    the start of the call are served first, then the others, ascending inside each class; a
    cache of n_slots whole entries, least recently used slot replaced."""
    lru, copies = [], []          # most recently used last
    for entries in batches_of_entries:
        distinct = sorted(set(entries))
        c = 0
        for e in [e for e in distinct if e in lru] + [e for e in distinct if e not in lru]:
            if e in lru:
                lru.remove(e)
            else:
                c += 1
                if len(lru) == n_slots:
                    lru.pop(0)
            lru.append(e)
        copies.append(c)
    return copies


def test_workload_5_host_resident_store_at_the_pinned_limit_all_256_searches_all_262144_tiles(env, oracle_mod):
    """Over-HBM workload: 1,000,000 x 256 index in HBM, map store in pinned host memory at the
    largest size the box grants, streamed by hipMemcpyAsync on a side stream.  Two batches of 256
    queries (Zipf(1.1) popularity): the first is checked in full (all 256 searches, every one of
    its 256 x 32 x 32 output tiles), the second exercises the entry cache across batches (96
    slots: fewer than a batch's distinct entries, so slots are also recycled inside a batch) and
    is checked on every tile of every eighth query; copy counts must equal the LRU policy's."""
    ac, synth, synthdb = env
    dev = torch.device("cuda:0")
    store = None
    for n_entries in HOST_ENTRY_LADDER:
        w = synth.WORKLOADS[5].scaled(n_entries=n_entries)
        try:
            store = synthdb.SynthMapStore(w, dev, layout="packed", host=True)
            break
        except MemoryError as e:
            print(f"[workload 5] {e}; trying fewer entries", flush=True)
    assert store is not None, "no pinned host memory for even the smallest store"
    print(f"[workload 5] host store: {w.n_entries} entries, {store.stored_bytes / 2**30:.1f} GiB pinned",
          flush=True)
    B, L, Hq, Hkv, S, D = w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    emb, raw, map_of = synth.make_embeddings(w, dev)
    Q, K, V = synth.make_qkv(w, dev)
    del Q, K
    entry_bytes = store.stored_bytes // w.n_entries
    n_slots = 96
    staging = torch.empty(n_slots * entry_bytes, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    db = ac.attncache_build_db(emb, store.maps, n_kv_heads=Hkv, head_dim=D, causal=w.causal,
                               map_of=map_of, seq_len=S, staging=staging, side_stream=side)
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, w.k), dtype=torch.uint8, device=dev)
    idx = torch.empty(B, w.k, dtype=torch.int32, device=dev)
    score = torch.empty(B, w.k, dtype=torch.float32, device=dev)
    hit = torch.empty(B, dtype=torch.int32, device=dev)
    O = torch.empty(B, L, Hq, S, D, dtype=torch.bfloat16, device=dev)
    seen, total_tiles = [], 0
    for batch_id in (0, 1):
        q, planted = synth.make_queries(w, raw, dev, batch_id=batch_id)
        O.fill_(3.0)
        ac.attncache_search(db, q, w.k, w.theta, idx, score, hit, ws)
        hit_host = hit.cpu()                      # the host schedules the copies
        ac.attncache_apply(db, hit_host, V, O)
        torch.cuda.synchronize()
        hit_h = hit_host.numpy()
        assert np.array_equal(hit_h, (planted % w.n_entries).numpy().astype(np.int32))
        seen.append([int(e) for e in hit_h])
        if batch_id == 0:
            assert parity.check_search(oracle_mod, q, emb, w.k, w.theta, 0, map_of, idx, score, hit) <= 2
            queries = list(range(B))
        else:
            queries = list(range(0, B, 8))
        total_tiles += _check_reuse_tiles(oracle_mod, store, hit_h, V, O, queries, 2e-2)
        lookups, copies = ac.attncache_cache_stats(db)
        want = _lru_copies(seen, n_slots)
        assert lookups == sum(len(set(s)) for s in seen) and copies == sum(want), (lookups, copies, want)
        print(f"[workload 5] batch {batch_id}: {len(set(seen[-1]))} distinct entries, "
              f"{want[-1]} copied", flush=True)
    assert total_tiles == (256 + 32) * 32 * 32
    assert len(set(seen[0])) > n_slots            # slots were recycled inside the first batch
    assert _lru_copies(seen, n_slots)[1] < len(set(seen[1]))   # and the second batch found entries cached
    db.close()
    store.close()


@pytest.mark.parametrize("cfg", [2, 4], ids=["llama-1b-shape", "long-sequence-shape"])
def test_insert_and_projector_at_full_batch_size(env, oracle_mod, cfg):
    """Database building at a workload's full batch shape: every item of the batch is computed,
    remembered (packed layout) and found again; the oracle checks sampled tiles of the stored
    maps and of the outputs, and the features come from the projector at the model's width."""
    ac, synth, _ = env
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[cfg]
    B, L, Hq, Hkv, S, D, E = (w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim,
                              w.emb_dim)
    g = Hq // Hkv
    M = B + 3
    Q, K, V = synth.make_qkv(w, dev)

    # features: projector on synthetic hidden states of the model's width
    dm, hid = Hq * D, Hq * D // 4
    gen = torch.Generator(device=dev).manual_seed(synth.seed_for(w, 9))
    h = (torch.randn(B, 1, dm, generator=gen, device=dev) +
         torch.randn(B, S, dm, generator=gen, device=dev)).to(torch.bfloat16)
    W1 = torch.randn(hid, dm, generator=gen, device=dev) / dm ** 0.5
    W2 = torch.randn(E, hid, generator=gen, device=dev) / hid ** 0.5
    b1 = 0.1 * torch.randn(hid, generator=gen, device=dev)
    b2 = 0.1 * torch.randn(E, generator=gen, device=dev)
    pws = torch.empty(ac.attncache_project_workspace_bytes(B, dm, hid, E), dtype=torch.uint8, device=dev)
    feat = torch.empty(B, E, dtype=torch.float16, device=dev)
    ac.attncache_project(h, W1, b1, W2, b2, feat, pws)
    torch.cuda.synchronize()
    rows = [0, B // 2, B - 1]
    want = oracle_mod.project(parity.to_np(h[rows]), parity.to_np(W1), parity.to_np(b1),
                              parity.to_np(W2), parity.to_np(b2))
    assert np.abs(parity.to_np(feat[rows]) - want).max() <= 2e-5 + 2.0 ** -11

    # an empty database of M slots; the batch takes slots in a scrambled order
    tile = ac.packed_tile_elems(S, w.causal)
    maps = torch.zeros(M, L, Hq, tile, dtype=torch.bfloat16, device=dev)
    emb = torch.zeros(M, E, dtype=torch.float16, device=dev)
    db = ac.attncache_build_db(emb, maps, n_kv_heads=Hkv, head_dim=D, causal=w.causal, seq_len=S)
    slot = torch.randperm(M, generator=torch.Generator().manual_seed(cfg))[:B].int().to(dev)
    O = torch.full((B, L, Hq, S, D), 3.0, dtype=torch.bfloat16, device=dev)
    ac.attncache_insert(db, Q, K, V, O, slot=slot, feat=feat)
    torch.cuda.synchronize()
    assert torch.isfinite(O.view(-1)[:: max(1, O.numel() // (1 << 24))].float()).all()

    slot_h = slot.cpu().numpy()
    for (b, l, hq) in _sample_tiles(list(range(B)), L, Hq, 6, cfg + 300):
        ref_O, P = oracle_mod.attention_exact(parity.to_np(Q[b, l, hq]).reshape(1, 1, S, D),
                                              parity.to_np(K[b, l, hq // g]).reshape(1, 1, S, D),
                                              parity.to_np(V[b, l, hq // g]).reshape(1, 1, S, D),
                                              causal=w.causal, return_map=True)
        assert parity.max_abs_err(O[b, l, hq].contiguous(), ref_O[0, 0]) <= 2e-2, (b, l, hq)
        stored = parity.unpack_map(parity.to_np(maps[int(slot_h[b]), l, hq]), S, w.causal)
        parity.check_stored_map(stored, oracle_mod.round_maps(P, oracle_mod.ROUND_BF16)[0, 0])

    # the same inputs now hit their own slots, and the reuse branch returns what was computed
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, 1), dtype=torch.uint8, device=dev)
    idx = torch.empty(B, 1, dtype=torch.int32, device=dev)
    score = torch.empty(B, 1, dtype=torch.float32, device=dev)
    hit = torch.empty(B, dtype=torch.int32, device=dev)
    ac.attncache_search(db, feat, 1, 0.99, idx, score, hit, ws)
    O2 = torch.full_like(O, 5.0)
    ac.attncache_apply(db, hit, V, O2)
    torch.cuda.synchronize()
    assert torch.equal(hit, slot)
    assert float((O2.float() - O.float()).abs().max()) <= 2e-2
    unused = sorted(set(range(M)) - set(int(x) for x in slot_h))
    assert torch.count_nonzero(maps[unused]) == 0 and torch.count_nonzero(emb[unused]) == 0
    db.close()
