"""Helpers shared by the GPU parity tests: run one step on the GPU library and on the oracle
with the same bytes, and compare to the stated bars.

Bars (stated once, used everywhere):
  * indices: bit-exact; a rank is exempt only when the oracle's fp32 score at that rank is
    within 1e-5 (relative) of a neighbouring rank's score (rank k is compared with rank k+1),
    and even then the GPU's row must score within 1e-5 of the oracle's score at that rank;
  * scores: 1e-5 relative (fp32 accumulation order differs);
  * hit: exact, unless the best similarity is within 1e-5 relative of the threshold;
  * outputs: max-abs error against the UNROUNDED fp64 oracle <= 2e-2 for bf16 data,
    <= 1e-4 for fp32 data.
"""
import numpy as np
import torch

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}
REL_TIE = 1e-5


def to_np(t: torch.Tensor) -> np.ndarray:
    """Exact fp32 copy of a (possibly bf16 / fp16, possibly CUDA) tensor on the host."""
    return t.detach().to("cpu", torch.float32).numpy()


def check_search(oracle, q, emb, k, theta, metric, map_of, gpu_idx, gpu_score, gpu_hit):
    """Compare search results with the oracle.  Returns the number of exempted ranks."""
    qn, en = to_np(q), to_np(emb)
    N = en.shape[0]
    kk = min(k + 1, N)
    mo = None if map_of is None else map_of.cpu().numpy()
    o_idx, o_score, _ = oracle.search(qn, en, k=kk, theta=theta, metric=metric, map_of=mo)
    _, _, o_hit = oracle.search(qn, en, k=1, theta=theta, metric=metric, map_of=mo)
    g_idx, g_score, g_hit = gpu_idx.cpu().numpy(), gpu_score.cpu().numpy(), gpu_hit.cpu().numpy()
    exempt = 0
    B = qn.shape[0]
    for b in range(B):
        for r in range(k):
            s = float(o_score[b, r])
            tol = REL_TIE * max(abs(s), 1e-30)
            assert abs(float(g_score[b, r]) - s) <= tol, (b, r, g_score[b, r], s)
            if g_idx[b, r] == o_idx[b, r]:
                continue
            near = []
            if r > 0:
                near.append(abs(float(o_score[b, r - 1]) - s))
            if r + 1 < kk:
                near.append(abs(float(o_score[b, r + 1]) - s))
            assert near and min(near) <= tol, ("index mismatch without a near-tie", b, r,
                                               g_idx[b, r], o_idx[b, r])
            # the row the GPU named must itself score (in fp64) like the oracle's row
            row = en[g_idx[b, r]].astype(np.float64)
            qq = qn[b].astype(np.float64)
            true = float(qq @ row) if metric == 0 else -float(((qq - row) ** 2).sum())
            assert abs(true - s) <= 2 * tol, (b, r)
            exempt += 1
        best = float(o_score[b, 0])
        sim = best if metric == 0 else 1.0 - float(np.sqrt(max(-best, 0.0)))
        if abs(sim - theta) <= REL_TIE * max(abs(theta), 1e-30):
            exempt += 1
            continue
        if g_idx[b, 0] == o_idx[b, 0]:
            assert g_hit[b] == o_hit[b], (b, g_hit[b], o_hit[b])
        else:
            assert (g_hit[b] >= 0) == (o_hit[b] >= 0), b
    return exempt


def max_abs_err(gpu_out: torch.Tensor, oracle_out: np.ndarray) -> float:
    g = gpu_out.detach().to("cpu", torch.float64).numpy()
    assert g.shape == oracle_out.shape
    assert np.isfinite(g).all()
    return float(np.abs(g - oracle_out).max())
