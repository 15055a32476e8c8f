"""attncache_search_static (the entry point that allocates nothing: its workspace is an array
inside the library) against attncache_search with a caller-provided workspace, through the C ABI.
Both run the same kernels, so every output must be bit-identical; attncache_search itself is
compared with the oracle elsewhere.  Two calls in a row share the array, the second with a
smaller input."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ac():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    from paper_2510_25979_amd import binding
    binding.lib()
    return binding


def _unit(x):
    return x / x.norm(dim=-1, keepdim=True)


def _db(ac, N, E, seed, dtype=torch.float16):
    g = torch.Generator(device="cuda").manual_seed(seed)
    emb = _unit(torch.randn(N, E, generator=g, device="cuda")).to(dtype)
    maps = torch.zeros(8, 1, 1, 32, 32, dtype=torch.bfloat16, device="cuda")
    map_of = (torch.arange(N, device="cuda") % 8).int()
    return emb, ac.attncache_build_db(emb, maps, n_kv_heads=1, head_dim=64, map_of=map_of), g


def _both(ac, db, q, k, theta):
    """(idx, score, hit) from the static-workspace entry point and from the ordinary one."""
    B = q.shape[0]
    out = []
    for static in (True, False):
        idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
        score = torch.full((B, k), -7.0, dtype=torch.float32, device="cuda")
        hit = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        if static:
            ac.attncache_search_static(db, q, k, theta, idx, score, hit)
        else:
            ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, k), dtype=torch.uint8, device="cuda")
            ac.attncache_search(db, q, k, theta, idx, score, hit, ws)
        torch.cuda.synchronize()
        out.append((idx, score, hit))
    return out


@pytest.mark.parametrize("N,E,k,B1,B2", [
    (70_001, 256, 1, 130, 37),     # query-stationary kernel, ragged last group and last chunk
    (5_000, 128, 4, 48, 5),        # row-stationary kernel, top-4 (candidate area in use)
    (3_000, 96, 3, 9, 2),          # width the matrix-core kernels are not built for
], ids=["N70001-E256-k1-B130-then-37", "N5000-E128-k4-B48-then-5", "N3000-E96-k3-B9-then-2"])
def test_static_workspace_search_equals_search_twice_in_a_row(ac, N, E, k, B1, B2):
    emb, db, g = _db(ac, N, E, 77 + N)
    for B in (B1, B2):             # the second, smaller call finds the first one's leftovers
        rows = torch.randint(0, N, (B,), generator=g, device="cuda")
        q = _unit(emb[rows].float() + 0.02 * torch.randn(B, E, generator=g, device="cuda")).half()
        q[B // 2] = _unit(torch.randn(E, generator=g, device="cuda")).half()      # a miss
        (i_s, s_s, h_s), (i_r, s_r, h_r) = _both(ac, db, q, k, 0.9)
        assert torch.equal(i_s, i_r) and torch.equal(h_s, h_r)
        assert torch.equal(s_s.view(torch.int32), s_r.view(torch.int32))          # bit-identical
        assert torch.equal(i_r[:, 0].long() == rows, h_r >= 0)                    # planted found, miss missed
        assert int((h_r < 0).sum()) == 1
    db.close()


def test_static_workspace_search_fp32_l2(ac):
    g = torch.Generator(device="cuda").manual_seed(5)
    emb = torch.randn(1500, 40, generator=g, device="cuda")
    maps = torch.zeros(1500, 1, 1, 8, 8, dtype=torch.float32, device="cuda")
    db = ac.attncache_build_db(emb, maps, n_kv_heads=1, head_dim=8, metric=ac.AC_L2)
    for B in (11, 3):
        q = emb[torch.randint(0, 1500, (B,), generator=g, device="cuda")] + \
            0.01 * torch.randn(B, 40, generator=g, device="cuda")
        (i_s, s_s, h_s), (i_r, s_r, h_r) = _both(ac, db, q, 2, 0.5)
        assert torch.equal(i_s, i_r) and torch.equal(h_s, h_r) and torch.equal(s_s, s_r)
        assert (h_r >= 0).all()
    db.close()


def test_static_workspace_search_rejects_what_does_not_fit(ac):
    # 64 candidates x 1024 rows x 4 bytes per query: 600 queries need far more than the 4 MiB array
    emb, db, g = _db(ac, 200_000, 128, 3)
    B, k = 600, 64
    assert ac.attncache_workspace_bytes(db.desc, B, k) > ac.AC_STATIC_SCRATCH_BYTES
    q = emb[:B].contiguous()
    idx = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    score = torch.zeros(B, k, device="cuda")
    hit = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(ac.AttnCacheError) as e:
        ac.attncache_search_static(db, q, k, 0.9, idx, score, hit)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert (idx == -7).all() and (hit == -7).all()          # nothing was launched
    # raw C ABI: NULL handle and an empty batch
    L = ac.lib()
    assert L.attncache_search_static(None, None, 1, 1, ctypes.c_float(0.0), None, None, None, None) == -1
    assert L.attncache_search_static(db.handle, None, 0, 1, ctypes.c_float(0.0), None, None, None, None) == 0
    db.close()
