"""GPU parity of the feature projector (Algorithm 1: f = feature_projector(h)) against the CPU
oracle, through the C ABI.

Bar: all arithmetic is binary32; a dot product of K terms with fp32 accumulation is within about
sqrt(K) * 2^-24 of its exact value relative to the size of its terms, and the two layers
chain two of them, so an unrounded (fp32) output must be within 2e-5 * max(1, max |f[b]|) of the
fp64 oracle.  An fp16 output adds the one rounding to half precision: half a unit in the last
place, 2^-11 relative.
"""
import numpy as np
import pytest
import torch

from tests import parity

pytestmark = pytest.mark.gpu

ABS = 2e-5
HALF_ULP_F16 = 2.0 ** -11


@pytest.fixture(scope="module")
def ac():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    from paper_2510_25979_amd import binding
    binding.lib()
    return binding


def _inputs(seed, B, S, dm, hid, E, h_dtype, biases=True):
    """Hidden states with a per-sentence offset (so that the token mean is not ~0), weights scaled
    by 1/sqrt(fan-in) like a freshly initialised linear layer."""
    g = torch.Generator().manual_seed(seed)
    h = (torch.randn(B, 1, dm, generator=g) + torch.randn(B, S, dm, generator=g)).to(h_dtype)
    W1 = torch.randn(hid, dm, generator=g) / dm ** 0.5
    W2 = torch.randn(E, hid, generator=g) / hid ** 0.5
    b1 = 0.1 * torch.randn(hid, generator=g) if biases else None
    b2 = 0.1 * torch.randn(E, generator=g) if biases else None
    return h, W1, b1, W2, b2


def _run(ac, h, W1, b1, W2, b2, feat_dtype, seq_len=None, normalize=True):
    B, S, dm = h.shape
    hid, E = W1.shape[0], W2.shape[0]
    dev = lambda t: None if t is None else t.cuda()
    ws = torch.empty(ac.attncache_project_workspace_bytes(B, dm, hid, E), dtype=torch.uint8,
                     device="cuda")
    ws.fill_(0xFF)                                   # scratch arrives dirty (NaN patterns)
    feat = torch.full((B, E), 7.0, dtype=feat_dtype, device="cuda")
    ac.attncache_project(dev(h), dev(W1), dev(b1), dev(W2), dev(b2), feat, ws,
                         seq_len=dev(seq_len), normalize=normalize)
    torch.cuda.synchronize()
    return feat


def _check(oracle_mod, got, h, W1, b1, W2, b2, seq_len, normalize):
    n = lambda t: None if t is None else parity.to_np(t)
    sl = None if seq_len is None else seq_len.numpy()
    want = oracle_mod.project(n(h), n(W1), n(b1), n(W2), n(b2), seq_len=sl, normalize=normalize)
    g = parity.to_np(got).astype(np.float64)
    scale = np.maximum(1.0, np.abs(want).max(axis=1, keepdims=True))
    tol = ABS * scale
    if got.dtype == torch.float16:
        tol = tol + HALF_ULP_F16 * np.abs(want)
    err = np.abs(g - want)
    assert np.all(err <= tol), (float((err / tol).max()), np.unravel_index((err / tol).argmax(), err.shape))
    return want


CASES = [
    # B, S, dm, hid, E, h dtype, feat dtype, ragged lengths, normalize, biases
    (64, 128, 2048, 512, 256, torch.bfloat16, torch.float16, False, True, True),   # 1B-shaped, workload 2's batch
    (5, 37, 72, 40, 24, torch.float32, torch.float32, True, False, True),          # every edge ragged
    (33, 50, 264, 136, 128, torch.bfloat16, torch.float32, True, True, False),     # 2 query tiles, no biases
    (70, 16, 4096, 1024, 128, torch.bfloat16, torch.float16, True, True, True),    # 8B-shaped width, 3 query tiles
    (1, 1, 8, 8, 8, torch.float32, torch.float32, False, False, True),             # smallest sizes accepted
    (130, 9, 520, 264, 2048, torch.bfloat16, torch.float32, True, True, True),     # widest feature vector
    (3, 1000, 264, 136, 64, torch.bfloat16, torch.float16, True, True, True),      # long sentences: several pooling rounds
    (2, 300, 128, 64, 32, torch.float32, torch.float32, False, False, True),       # the same with fp32 hidden states
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "B%d_S%d_dm%d_hid%d_E%d" % c[:5])
def test_projector_matches_oracle(ac, oracle_mod, case):
    B, S, dm, hid, E, hdt, fdt, ragged, normalize, biases = case
    h, W1, b1, W2, b2 = _inputs(4100 + B, B, S, dm, hid, E, hdt, biases)
    seq_len = None
    if ragged:
        seq_len = torch.randint(1, S + 1, (B,), generator=torch.Generator().manual_seed(B)).int()
        seq_len[0], seq_len[-1] = S, 1
        for b in range(B):                            # tokens past the end must not be read into the mean
            h[b, seq_len[b]:] = 1e4
    got = _run(ac, h, W1, b1, W2, b2, fdt, seq_len, normalize)
    want = _check(oracle_mod, got, h, W1, b1, W2, b2, seq_len, normalize)
    if normalize:
        np.testing.assert_allclose(np.linalg.norm(want, axis=1), 1.0, rtol=1e-12)


def test_projector_closed_form_and_clamped_lengths(ac, oracle_mod):
    # signed identity layers: f = relu(x) - relu(-x) = x, so the output is the token mean itself
    B, S, dm = 6, 20, 64
    g = torch.Generator().manual_seed(9)
    h = torch.randn(B, S, dm, generator=g)
    eye = torch.eye(dm)
    W1, W2 = torch.cat([eye, -eye], 0), torch.cat([eye, -eye], 1)
    seq_len = torch.tensor([0, 25, 7, 20, 1, -3], dtype=torch.int32)     # 0, 25, -3 are clamped to 1, 20, 1
    clamped = seq_len.clamp(1, S)
    got = _run(ac, h, W1, None, W2, None, torch.float32, seq_len, normalize=False)
    mean = torch.stack([h[b, :clamped[b]].double().mean(0) for b in range(B)])
    assert float((got.cpu().double() - mean).abs().max()) <= 1e-6
    _check(oracle_mod, got, h, W1, None, W2, None, clamped, False)
    # a zero feature vector stays zero under normalisation
    z = _run(ac, h, torch.zeros(16, dm), None, torch.ones(8, 16), None, torch.float16, None, True)
    assert torch.count_nonzero(z) == 0


def test_projector_is_deterministic_and_feeds_search(ac, oracle_mod):
    # database features and query features both come from the projector; the planted neighbour
    # of each query must be found, and search on those bytes must equal the oracle's search
    N, B, S, dm, hid, E = 300, 40, 24, 256, 128, 64
    h_db, W1, b1, W2, b2 = _inputs(77, N, S, dm, hid, E, torch.bfloat16)
    emb = _run(ac, h_db, W1, b1, W2, b2, torch.float16)
    again = _run(ac, h_db, W1, b1, W2, b2, torch.float16)
    assert torch.equal(emb, again)
    g = torch.Generator().manual_seed(78)
    rows = torch.randperm(N, generator=g)[:B]
    h_q = (h_db[rows].float() + 0.02 * torch.randn(B, S, dm, generator=g)).to(torch.bfloat16)
    q = _run(ac, h_q, W1, b1, W2, b2, torch.float16)
    maps = torch.zeros(N, 1, 1, 32, 32, dtype=torch.bfloat16, device="cuda")
    db = ac.attncache_build_db(emb, maps, n_kv_heads=1, head_dim=64)
    ws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, 2), dtype=torch.uint8, device="cuda")
    idx = torch.empty(B, 2, dtype=torch.int32, device="cuda")
    score = torch.empty(B, 2, device="cuda")
    hit = torch.empty(B, dtype=torch.int32, device="cuda")
    ac.attncache_search(db, q, 2, 0.9, idx, score, hit, ws)
    torch.cuda.synchronize()
    parity.check_search(oracle_mod, q, emb, 2, 0.9, 0, None, idx, score, hit)
    assert torch.equal(idx[:, 0].cpu().long(), rows)
    assert torch.equal(hit.cpu().long(), rows)
    db.close()


def test_projector_and_search_replayed_from_a_hip_graph(ac):
    N, B, S, dm, hid, E = 200, 16, 32, 128, 64, 64
    _, W1, b1, W2, b2 = _inputs(5, 1, S, dm, hid, E, torch.bfloat16)
    W1, b1, W2, b2 = (t.cuda() for t in (W1, b1, W2, b2))
    emb = torch.nn.functional.normalize(torch.randn(N, E, generator=torch.Generator().manual_seed(6)),
                                        dim=-1).half().cuda()
    maps = torch.zeros(N, 1, 1, 32, 32, dtype=torch.bfloat16, device="cuda")
    db = ac.attncache_build_db(emb, maps, n_kv_heads=1, head_dim=64)
    h = torch.empty(B, S, dm, dtype=torch.bfloat16, device="cuda")
    pws = torch.empty(ac.attncache_project_workspace_bytes(B, dm, hid, E), dtype=torch.uint8, device="cuda")
    sws = torch.empty(ac.attncache_workspace_bytes(db.desc, B, 1), dtype=torch.uint8, device="cuda")
    feat = torch.empty(B, E, dtype=torch.float16, device="cuda")
    idx = torch.empty(B, 1, dtype=torch.int32, device="cuda")
    score = torch.empty(B, 1, device="cuda")
    hit = torch.empty(B, dtype=torch.int32, device="cuda")

    def step():
        ac.attncache_project(h, W1, b1, W2, b2, feat, pws)
        ac.attncache_search(db, feat, 1, 0.0, idx, score, hit, sws)

    h.copy_(torch.randn(B, S, dm, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16))
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for seed in (2, 3, 4):
        h.copy_(torch.randn(B, S, dm, generator=torch.Generator().manual_seed(seed)).to(torch.bfloat16))
        graph.replay()
        torch.cuda.synchronize()
        got = (feat.clone(), idx.clone(), score.clone())
        feat.zero_(); idx.zero_(); score.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got[0], feat) and torch.equal(got[1], idx) and torch.equal(got[2], score)
    db.close()


def test_projector_error_codes(ac):
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device="cuda")
    h, W1, W2 = z(2, 4, 16, dt=torch.bfloat16), z(8, 16), z(8, 8)
    feat = z(2, 8, dt=torch.float16)
    ws = torch.zeros(ac.attncache_project_workspace_bytes(2, 16, 8, 8), dtype=torch.uint8, device="cuda")
    ac.attncache_project(h, W1, None, W2, None, feat, ws)                 # accepted as is
    ac.attncache_project(h[:0], W1, None, W2, None, feat[:0], ws)         # empty batch: nothing to do
    with pytest.raises(ac.AttnCacheError) as e:                           # workspace too small
        ac.attncache_project(h, W1, None, W2, None, feat, ws[:64])
    assert e.value.status == -6
    with pytest.raises(ac.AttnCacheError) as e:                           # misaligned workspace
        ac.attncache_project(h, W1, None, W2, None, feat, torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")[4:])
    assert e.value.status == -4
    with pytest.raises(ac.AttnCacheError) as e:                           # width not a multiple of 8
        ac.attncache_project(z(2, 4, 12, dt=torch.bfloat16), z(8, 12), None, W2, None, feat, ws)
    assert e.value.status == -2
    with pytest.raises(ac.AttnCacheError) as e:                           # feature vector too wide
        ac.attncache_project(h, W1, None, z(2056, 8), None, z(2, 2056, dt=torch.float16), ws)
    assert e.value.status == -2
    import ctypes
    L = ac.lib()
    rc = L.attncache_project(h.data_ptr(), None, W1.data_ptr(), None, W2.data_ptr(), None,
                             feat.data_ptr(), 2, 4, 16, 8, 8, ac.AC_F16, ac.AC_F16, 1,
                             ws.data_ptr(), ctypes.c_size_t(ws.numel()), None)
    assert rc == -3                                                       # fp16 hidden states are not supported
    rc = L.attncache_project(h.data_ptr(), None, None, None, W2.data_ptr(), None,
                             feat.data_ptr(), 2, 4, 16, 8, 8, ac.AC_BF16, ac.AC_F16, 1,
                             ws.data_ptr(), ctypes.c_size_t(ws.numel()), None)
    assert rc == -1
    assert ac.attncache_project_workspace_bytes(0, 16, 8, 8) == 0
    torch.cuda.synchronize()
