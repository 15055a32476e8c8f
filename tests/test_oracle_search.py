"""Pins for the oracle's search (Algorithm 1: VecDB.search + threshold test).

Each test checks the oracle against something fixed outside it: a hand-worked case, a closed
form, an invariant, or a library routine.
"""
import numpy as np
import pytest
import torch

from paper_2510_25979_amd import synth


def test_hand_worked_inner_products(oracle_mod):
    # <q,e> by hand: rows give 1*1+2*0=1, 1*0+2*1=2, 1*1+2*1=3, -1-2=-3
    emb = np.array([[1, 0], [0, 1], [1, 1], [-1, -1]], np.float32)
    q = np.array([[1, 2]], np.float32)
    idx, score, hit = oracle_mod.search(q, emb, k=4, theta=2.5)
    assert idx.tolist() == [[2, 1, 0, 3]]
    assert score.tolist() == [[3.0, 2.0, 1.0, -3.0]]
    assert hit.tolist() == [2]
    # transposed-operand trap: a non-square problem where q and emb cannot be swapped
    q2 = np.array([[1, 2], [0, -1], [3, 0]], np.float32)
    idx, score, _ = oracle_mod.search(q2, emb, k=1)
    assert idx[:, 0].tolist() == [2, 3, 0] and score[:, 0].tolist() == [3.0, 1.0, 3.0]


def test_hand_worked_l2(oracle_mod):
    emb = np.array([[0, 0], [3, 4], [1, 0]], np.float32)
    q = np.array([[0, 0.5]], np.float32)
    idx, score, hit = oracle_mod.search(q, emb, k=3, theta=0.4, metric=oracle_mod.METRIC_L2)
    # squared distances 0.25, 9+12.25=21.25, 1.25 -> scores are their negatives
    assert idx.tolist() == [[0, 2, 1]]
    assert score.tolist() == [[-0.25, -1.25, -21.25]]
    assert hit.tolist() == [0]          # similarity 1 - 0.5 = 0.5 >= 0.4
    _, _, hit = oracle_mod.search(q, emb, k=1, theta=0.6, metric=oracle_mod.METRIC_L2)
    assert hit.tolist() == [-1]         # 0.5 < 0.6


def test_identity_database_gives_largest_components(oracle_mod):
    rng = np.random.default_rng(1)
    E = 37
    q = rng.standard_normal((5, E)).astype(np.float32)
    idx, score, _ = oracle_mod.search(q, np.eye(E, dtype=np.float32), k=6)
    for b in range(5):
        order = np.argsort(-q[b], kind="stable")[:6]
        assert idx[b].tolist() == order.tolist()
        assert np.array_equal(score[b], q[b][order])


def test_duplicates_rank_lowest_index_first(oracle_mod):
    rng = np.random.default_rng(2)
    emb = rng.standard_normal((50, 16)).astype(np.float32)
    emb[[7, 19, 33]] = emb[3]          # four identical rows: 3, 7, 19, 33
    q = (emb[3] * 4).reshape(1, -1)
    idx, score, _ = oracle_mod.search(q, emb, k=4)
    assert idx.tolist() == [[3, 7, 19, 33]]
    assert len(set(score[0].tolist())) == 1


def test_row_permutation_permutes_indices_only(oracle_mod):
    rng = np.random.default_rng(3)
    emb = rng.standard_normal((200, 24)).astype(np.float32)
    q = rng.standard_normal((6, 24)).astype(np.float32)
    perm = rng.permutation(200)
    i0, s0, _ = oracle_mod.search(q, emb, k=5)
    i1, s1, _ = oracle_mod.search(q, emb[perm], k=5)
    assert np.array_equal(perm[i1], i0)
    assert np.array_equal(s0, s1)


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_against_library_topk(oracle_mod, metric):
    g = torch.Generator().manual_seed(4)
    emb = torch.randn(777, 48, generator=g, dtype=torch.float64).float()
    q = torch.randn(9, 48, generator=g, dtype=torch.float64).float()
    if metric == "ip":
        ref = q.double() @ emb.double().T
        m = oracle_mod.METRIC_IP
    else:
        ref = -(torch.cdist(q.double(), emb.double()) ** 2)
        m = oracle_mod.METRIC_L2
    top = torch.topk(ref, 8, dim=1)
    idx, score, _ = oracle_mod.search(q.numpy(), emb.numpy(), k=8, metric=m)
    assert np.array_equal(idx, top.indices.numpy().astype(np.int32))
    np.testing.assert_allclose(score, top.values.numpy(), rtol=2e-7, atol=1e-9)


def test_threshold_is_not_less_than(oracle_mod):
    emb = np.eye(4, dtype=np.float32)
    q = np.array([[0, 0, 1, 0]], np.float32)          # best score is exactly 1.0
    assert oracle_mod.search(q, emb, theta=1.0)[2].tolist() == [2]
    above = float(np.nextafter(np.float32(1.0), np.float32(2.0)))
    assert oracle_mod.search(q, emb, theta=above)[2].tolist() == [-1]
    below = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
    assert oracle_mod.search(q, emb, theta=below)[2].tolist() == [2]


def test_map_of_indirection(oracle_mod):
    emb = np.eye(6, dtype=np.float32)
    map_of = np.array([0, 1, 2, 0, 1, 2], np.int32)
    q = np.eye(6, dtype=np.float32)[[4, 5, 0]]
    idx, _, hit = oracle_mod.search(q, emb, theta=0.5, map_of=map_of)
    assert idx[:, 0].tolist() == [4, 5, 0]
    assert hit.tolist() == [1, 2, 0]


def test_planted_neighbour_is_recovered(oracle_mod):
    # the recipe of the workloads: a database row plus small noise must come back at rank 1
    for cfg, n in ((1, 1024), (2, 2000)):
        w = synth.WORKLOADS[cfg].scaled(n_emb=n, n_entries=n, batch=16)
        emb, raw, _ = synth.make_embeddings(w)
        q, planted = synth.make_queries(w, raw)
        idx, score, hit = oracle_mod.search(q.float().numpy(), emb.float().numpy(), k=2,
                                            theta=w.theta)
        assert np.array_equal(idx[:, 0], planted.numpy())
        assert np.array_equal(hit, planted.numpy())
        if w.normalise:
            assert score[:, 0].min() > 0.98 and score[:, 1].max() < 0.5


def test_half_planted_half_missing_routing(oracle_mod):
    w = synth.WORKLOADS[3].scaled(n_emb=1500, n_entries=1500, batch=32)
    emb, raw, _ = synth.make_embeddings(w)
    q, planted = synth.make_queries(w, raw)
    _, _, hit = oracle_mod.search(q.float().numpy(), emb.float().numpy(), theta=w.theta)
    assert (planted >= 0).sum().item() == 16
    assert np.array_equal(hit, planted.numpy())       # misses stay -1, hits name their row
    assert (hit >= 0).mean() == 0.5


def test_argument_errors(oracle_mod):
    emb = np.zeros((3, 2), np.float32)
    q = np.zeros((1, 2), np.float32)
    with pytest.raises(RuntimeError):
        oracle_mod.search(q, emb, k=4)
    with pytest.raises(RuntimeError):
        oracle_mod.search(q, emb, k=0)
