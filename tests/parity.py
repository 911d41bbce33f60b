"""Helpers shared by the GPU parity tests: run a stream through the C ABI and
compare with oracle outputs under the stated tolerances."""
import numpy as np
import torch

from oracle import proximity_oracle as po

ID_TIE_RTOL = 1e-5      # ids may differ only among rows whose distances agree to this
DIST_RTOL_F32 = 1e-4    # returned distances, float32 corpus
DIST_RTOL_BF16 = 2e-2   # returned distances, bfloat16 corpus


def run_stream(px, queries: np.ndarray, tau: float, batch: int, device):
    """Feed `queries` in order, `batch` rows per call.  Returns ids, dists, hit as numpy."""
    ids, dists, hit = [], [], []
    for b0 in range(0, len(queries), batch):
        q = torch.from_numpy(np.ascontiguousarray(queries[b0:b0 + batch])).to(device)
        i, d, h = px.search_batch(q, tau)
        ids.append(i)
        dists.append(d)
        hit.append(h)
    torch.cuda.synchronize(device)
    cat = lambda xs: torch.cat(xs).cpu().numpy()
    return cat(ids), cat(dists), cat(hit)


def assert_lists_match(ids, dists, o_ids, o_dists, corpus, ref_queries, dist_rtol=DIST_RTOL_F32, what="",
                       metric=po.METRIC_L2):
    """Row-wise comparison of ranked lists.

    `ref_queries[t]` is the vector the distances of row t refer to (the query
    itself on a miss, the matched key on a hit).  Ids must be equal; a row may
    differ from the oracle only by swapping or substituting documents whose
    float64 distances agree with the oracle's, position by position, to
    ID_TIE_RTOL.  Returned distances must be within dist_rtol.
    Returns the number of rows that needed the tie allowance.  `metric`: the index's distance
    function.  A cosine distance is evaluated as 1 - c with c near 1 and a negated inner product as a sum
    of terms of both signs, so a value near zero carries the absolute rounding error of its terms (a few
    1e-16 times |q||x| in float64, 6e-8 of the value once stored as float32) however small it is: for these
    two functions values are compared with an absolute allowance of 1e-12 beside the relative one.
    """
    atol = 0 if metric == po.METRIC_L2 else 1e-12
    assert ids.shape == o_ids.shape, what
    excused = 0
    bad_rows = np.flatnonzero((ids != o_ids).any(axis=1))
    for t in bad_rows:
        assert (ids[t] >= 0).all() == (o_ids[t] >= 0).all(), f"{what} row {t}: padding differs"
        valid = ids[t] >= 0
        assert (valid == (o_ids[t] >= 0)).all(), f"{what} row {t}: padding differs"
        assert len(set(ids[t][valid].tolist())) == valid.sum(), f"{what} row {t}: duplicate ids"
        d_true = po.metric_distances(ref_queries[t], corpus[ids[t][valid]], metric)
        np.testing.assert_allclose(d_true, o_dists[t][valid], rtol=ID_TIE_RTOL, atol=atol,
                                   err_msg=f"{what} row {t}: ids differ beyond near-ties")
        excused += 1
    fin = np.isfinite(o_dists)
    assert (np.isfinite(dists) == fin).all(), what
    np.testing.assert_allclose(dists[fin], o_dists[fin], rtol=dist_rtol, atol=atol, err_msg=what)
    return excused


def assert_stream_parity(gpu, oracle_out, corpus, queries, dist_rtol=DIST_RTOL_F32, what="", reranked=False,
                         metric=po.METRIC_L2):
    """`reranked`: the instance re-ranks on a hit (re-ranking factor above 1), so every row's
    distances refer to its own query; otherwise a hit row's distances refer to the matched key."""
    ids, dists, hit = gpu
    o_ids, o_dists, o_hit, o_src = oracle_out
    assert hit.dtype == np.uint8
    mism = np.flatnonzero(hit != o_hit)
    assert len(mism) == 0, f"{what}: hit/miss flags differ first at row {mism[:5]}"
    ref = np.asarray(queries) if reranked else np.asarray(queries)[o_src]
    return assert_lists_match(ids, dists, o_ids, o_dists, corpus, ref, dist_rtol, what, metric)
