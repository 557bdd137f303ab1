"""Reference scoring / ranking pass (numpy, fp64).  TEST INFRASTRUCTURE ONLY.

The task is a ranking problem over all entities [Sec. 3.2 "Objective
Function"]: f(q, e) = gamma - min_b ||y_b - Ef[e]||_1.  Smaller distance is
better; equal distances rank the lower entity id first.
"""
import numpy as np

from .model import dnf, forward, query_tree


def query_embeddings(batch, i, M):
    """[n_branches, d] branch embeddings of query i."""
    return np.stack([forward(b, M)[0] for b in dnf(query_tree(batch.query_nodes(i)))])


def score_candidates(batch, cand, M):
    """cand [B, C] entity ids -> scores [B, C]."""
    out = np.empty(cand.shape, np.float64)
    for i in range(batch.B):
        Y = query_embeddings(batch, i, M)
        rows = M.candidate(np.asarray(cand[i], np.int64))
        out[i] = M.gamma - np.abs(Y[:, None, :] - rows[None]).sum(axis=2).min(axis=0)
    return out


def distances_all(batch, i, M, chunk=8192):
    """L1 distance of query i to every entity, [N]."""
    Y = query_embeddings(batch, i, M)
    N = M.P["E"].shape[0]
    out = np.empty(N, np.float64)
    for lo in range(0, N, chunk):
        ids = np.arange(lo, min(N, lo + chunk))
        rows = M.candidate(ids)
        out[lo:lo + len(ids)] = np.abs(Y[:, None, :] - rows[None]).sum(axis=2).min(axis=0)
    return out


def topk_all(batch, i, M, k, distances=distances_all):
    """(ids, distances) of the k nearest entities: full sort, ties by id.  `distances` gives the
    distance of query i to every entity (the box family passes its own)."""
    dist = distances(batch, i, M)
    order = np.lexsort((np.arange(dist.shape[0]), dist))[:k]
    return order.astype(np.int64), dist[order]


def filtered_ranks(batch, i, answers, M, distances=distances_all):
    """Filtered rank of every listed answer of query i [the evaluation protocol behind the
    filtered MRR / Hit@k the paper reports, Sec. 5.3 and the large-KG table]: an answer's rank
    is 1 + the number of entities that are NOT listed answers of the query and lie strictly
    closer to the query than it does.  Returns (ranks [len(answers)], distances of the answers)."""
    dist = distances(batch, i, M)
    answers = np.asarray(answers, np.int64)
    other = np.ones(dist.shape[0], bool)
    other[answers] = False
    d_other = np.sort(dist[other])
    ranks = 1 + np.searchsorted(d_other, dist[answers], side="left")     # strictly smaller
    return ranks.astype(np.int64), dist[answers]


def ranking_metrics(rank_lists, ks=(1, 3, 10)):
    """Mean reciprocal rank and Hit@k: per query the mean over its ranked answers, then the
    mean over the queries that have at least one.  Returns [MRR, Hit@k1, Hit@k2, ...]."""
    per_query = []
    for r in rank_lists:
        r = np.asarray(r, np.float64)
        if r.size:
            per_query.append([np.mean(1.0 / r)] + [np.mean(r <= k) for k in ks])
    if not per_query:
        return np.zeros(1 + len(ks))
    return np.mean(np.asarray(per_query), axis=0)
