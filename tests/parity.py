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
            # fp32 accumulation error of an inner product is relative to its TERMS, sum |q_i e_i|
            # <= |q| |e| (Cauchy-Schwarz), not to the score, which cancellation can bring near
            # zero; the L2 score is a sum of non-negative terms and stays relative to itself
            scale = abs(s)
            if metric == 0:
                qq0 = qn[b].astype(np.float64)
                scale = max(scale, float(np.linalg.norm(qq0) * np.linalg.norm(en[o_idx[b, r]].astype(np.float64))))
            tol = REL_TIE * max(scale, 1e-30)
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


def unpack_map(packed: np.ndarray, S: int, causal: bool) -> np.ndarray:
    """Dense [S,S] view of one map stored in the block-packed layout the header documents
    (written here from that description, independently of the library): rows in blocks of 16,
    columns in blocks of 32; row block r keeps its first ceil((r+1)/2) column blocks (causal) or
    all of them; blocks row-block-major; inside a block element (i, 8q+e) sits at (16q+i)*8+e.
    Blocks that are not stored read as zeros."""
    out = np.zeros((S, S), packed.dtype)
    n32 = S // 32
    pos = 0
    for r in range(S // 16):
        nc = (r + 2) // 2 if causal else n32
        for cb in range(nc):
            blk = packed[pos:pos + 512].reshape(4, 16, 8)          # [q][i][e]
            out[16 * r:16 * r + 16, 32 * cb:32 * cb + 32] = blk.transpose(1, 0, 2).reshape(16, 32)
            pos += 512
    assert pos == packed.size
    return out


def check_stored_map(gpu_map: np.ndarray, oracle_map_rounded: np.ndarray):
    """A stored bf16 map against the oracle's map rounded to bf16.  The GPU forms the weights in
    fp32 (relative error ~1e-6) before the one rounding, the oracle in fp64: the two can land on
    neighbouring bf16 values when the exact weight lies next to a rounding boundary, never
    further apart.  Bar: every element within one bf16 ulp (2^-7 relative), at most 2 % of the
    elements different at all, zeros exactly zero."""
    g = gpu_map.astype(np.float64)
    r = oracle_map_rounded.astype(np.float64)
    assert g.shape == r.shape and np.isfinite(g).all()
    assert (g[r == 0.0] == 0.0).all()
    assert (np.abs(g - r) <= 2.0 ** -7 * np.maximum(np.abs(r), 1e-38)).all()
    assert (g != r).mean() <= 0.02
