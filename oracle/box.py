"""Box-embedding operator family: per-query reference of one training step (numpy, fp64).

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

The paper runs its framework over several operator parameterisations and names
the box model (Q2B) among them [Sec. 5.1 "Backbone models"]; it prints no
formulas.  The definitions below follow the published Query2Box model, with the
operator-level decomposition, objective and optimiser of oracle.model unchanged:

    state         a box (c, o): centre c and non-negative offset o, both width d
    anchor        (E[e], 0)
    projection    (c + R[r], o + relu(Ro[r]))                   no MLP
    intersection  centre: a_k = U2 relu(U1 c_k + u1) + u2; w = softmax over the k
                  inputs (per coordinate); c = sum_k w_k * c_k
                  offset: g = sigmoid(mean_k (V2 relu(V1 o_k + c1) + c2));
                  o = min_k o_k * g          (per coordinate; deep-set gate)
    union         disjunctive normal form; score = max over branches
    negation      not part of this family
    score         s(q,e) = gamma - min_b dist(box_b, E[e]),
                  dist = || relu(|e-c| - o) ||_1 + alpha * || min(|e-c|, o) ||_1
    loss, Adam    as in oracle.model; Ro is a row-sparse table like R
Kinks: relu'(0) = 0, sign(0) = 0, a coordinate with |e-c| == o counts as inside,
equal offsets in the min -> the lowest input, equal branch distances -> lowest branch.
"""
import numpy as np

from .model import (OP_NEG, Unsupported, adam_update, dnf, mlp_backward, mlp_forward, pair_loss_terms, query_tree,
                    sigmoid, to_f64)

TABLES = ("E", "R", "Ro")


class BoxModel:
    def __init__(self, params, gamma, alpha):
        self.P = to_f64(params)
        self.gamma = float(gamma)
        self.alpha = float(alpha)


class Grads:
    """Gradient accumulators; table gradients per touched row.  `mass` keeps, per row, the sum of
    the largest entries of its contributions: projections are translations here, so an entity that
    is an anchor of a query and one of its candidates receives two contributions that cancel, and
    the accuracy a sum of fp32 terms can have is set by the terms, not by what is left of them."""

    def __init__(self, P, track_sq=False):
        self.dense = {k: np.zeros_like(v) for k, v in P.items() if k not in TABLES}
        self.dense_sq = {k: np.zeros_like(v) for k, v in self.dense.items()} if track_sq else None   # as in oracle.model
        self.rows = {t: {} for t in TABLES}
        self.mass = {t: {} for t in TABLES}

    def add(self, name, val):
        self.dense[name] += val
        if self.dense_sq is not None:
            self.dense_sq[name] += np.square(val)

    def add_row(self, table, idx, vec):
        r = self.rows[table]
        idx = int(idx)
        r[idx] = r[idx] + vec if idx in r else np.array(vec, np.float64)
        self.mass[table][idx] = self.mass[table].get(idx, 0.0) + float(np.abs(vec).max())

    def table_dense(self, table, shape):
        out = np.zeros(shape, np.float64)
        for i, v in self.rows[table].items():
            out[i] = v
        return out


def forward(tree, M):
    """(centre, offset) of a conjunctive tree and what backward needs."""
    P = M.P
    kind = tree[0]
    if kind == "e":
        return P["E"][tree[1]], np.zeros(P["E"].shape[1]), ("e", tree[1])
    if kind == "p":
        c, o, tx = forward(tree[2], M)
        r = tree[1]
        return c + P["R"][r], o + np.maximum(P["Ro"][r], 0.0), ("p", r, tx)
    if kind == "i":
        cs, os_, txs, ctapes, otapes, att, gat = [], [], [], [], [], [], []
        for ch in tree[1:]:
            c, o, tx = forward(ch, M)
            a, tc = mlp_forward(c, P["U1"], P["u1"], P["U2"], P["u2"])
            g, to = mlp_forward(o, P["V1"], P["c1"], P["V2"], P["c2"])
            cs.append(c); os_.append(o); txs.append(tx); ctapes.append(tc); otapes.append(to)
            att.append(a); gat.append(g)
        C = np.stack(cs)
        O = np.stack(os_)
        A = np.stack(att)
        A = A - A.max(axis=0, keepdims=True)
        Wt = np.exp(A)
        Wt /= Wt.sum(axis=0, keepdims=True)
        gate = sigmoid(np.mean(np.stack(gat), axis=0))
        arg = np.argmin(O, axis=0)                      # first minimum
        omin = O[arg, np.arange(O.shape[1])]
        return (Wt * C).sum(axis=0), omin * gate, ("i", txs, ctapes, otapes, C, Wt, gate, arg, omin)
    if kind == "n":
        raise Unsupported("the box family has no negation")
    raise Unsupported("forward() takes conjunctive trees; split unions with dnf()")


def kink_margins(tape):
    """(smallest |pre-activation| of any hidden unit, smallest non-zero gap between the smallest
    and the second smallest input offset of an intersection) met while evaluating a tree: the
    distance of the evaluation from a ReLU kink and from a change of the arg-min."""
    kind = tape[0]
    if kind == "e":
        return np.inf, np.inf
    if kind == "p":
        return kink_margins(tape[2])
    _, txs, ctapes, otapes, C, Wt, gate, arg, omin = tape
    pre = min(float(np.abs(t[1]).min()) for t in ctapes + otapes)
    O = np.stack([t[0] for t in otapes])                # the inputs' offsets
    gaps = np.sort(O, axis=0)[1] - omin
    gap = float(gaps[gaps > 0].min()) if (gaps > 0).any() else np.inf
    for t in txs:
        p2, g2 = kink_margins(t)
        pre, gap = min(pre, p2), min(gap, g2)
    return pre, gap


def backward(tape, dc, do, M, G):
    P = M.P
    kind = tape[0]
    if kind == "e":
        G.add_row("E", tape[1], dc)                     # the anchor's offset is the constant 0
    elif kind == "p":
        _, r, tx = tape
        G.add_row("R", r, dc)
        G.add_row("Ro", r, do * (P["Ro"][r] > 0.0))
        backward(tx, dc, do, M, G)
    elif kind == "i":
        _, txs, ctapes, otapes, C, Wt, gate, arg, omin = tape
        k = C.shape[0]
        t_all = (Wt * C * dc).sum(axis=0)
        dpre = do * omin * gate * (1.0 - gate)          # gradient of the gate's pre-activation (a mean over k)
        for j in range(k):
            da = Wt[j] * (dc * C[j] - t_all)
            dca, dWa, dba, dWb, dbb = mlp_backward(da, ctapes[j], P["U1"], P["U2"])
            G.add("U1", dWa); G.add("u1", dba); G.add("U2", dWb); G.add("u2", dbb)
            doa, dWa, dba, dWb, dbb = mlp_backward(dpre / k, otapes[j], P["V1"], P["V2"])
            G.add("V1", dWa); G.add("c1", dba); G.add("V2", dWb); G.add("c2", dbb)
            backward(txs[j], Wt[j] * dc + dca, (arg == j) * do * gate + doa, M, G)
    else:
        raise ValueError(kind)


def box_distance(C, O, rows, alpha):
    """dist[b, m] of boxes (C[b], O[b]) to entity rows [m, d]."""
    a = np.abs(rows[None, :, :] - C[:, None, :])
    o = O[:, None, :]
    return np.maximum(a - o, 0.0).sum(axis=2) + alpha * np.minimum(a, o).sum(axis=2)


def score(C, O, rows, gamma, alpha):
    dist = box_distance(C, O, rows, alpha)
    win = np.argmin(dist, axis=0)
    return gamma - dist[win, np.arange(dist.shape[1])], win


def distances_all(batch, i, M, chunk=8192):
    """Box distance of query i to every entity (minimum over its branches), [N]."""
    fw = [forward(b, M) for b in dnf(query_tree(batch.query_nodes(i)))]
    C = np.stack([c for c, _, _ in fw])
    O = np.stack([o for _, o, _ in fw])
    N = M.P["E"].shape[0]
    out = np.empty(N, np.float64)
    for lo in range(0, N, chunk):
        hi = min(N, lo + chunk)
        out[lo:hi] = box_distance(C, O, M.P["E"][lo:hi], M.alpha).min(axis=0)
    return out


def query_step(nodes, pos, negs, M, B, G=None):
    if any(op == OP_NEG for op, _, _ in nodes):
        raise Unsupported("the box family has no negation")
    branches = dnf(query_tree(nodes))
    if any(b[0] == "e" for b in branches):
        raise Unsupported("a query must contain at least one operator")
    Cs, Os, tapes = [], [], []
    for b in branches:
        c, o, t = forward(b, M)
        Cs.append(c); Os.append(o); tapes.append(t)
    C, O = np.stack(Cs), np.stack(Os)
    cand = np.concatenate([[pos], np.asarray(negs, np.int64)])
    rows = M.P["E"][cand]
    s, win = score(C, O, rows, M.gamma, M.alpha)
    K = len(cand) - 1
    loss = pair_loss_terms(s[0], s[1:]) / (2.0 * B)
    if G is None:
        return loss, s
    coef = np.empty_like(s)
    coef[0] = -sigmoid(-s[0]) / (2.0 * B)
    coef[1:] = sigmoid(s[1:]) / (2.0 * B * K)
    dC, dO = np.zeros_like(C), np.zeros_like(O)
    for j in range(len(cand)):
        b = win[j]
        diff = C[b] - rows[j]
        outside = np.abs(diff) > O[b]
        w = np.where(outside, 1.0, M.alpha)             # d dist / d|e-c|
        # s = gamma - dist:  ds/dc = -w sign(c-e), ds/de = +w sign(c-e), ds/do = (1-alpha) [outside]
        dC[b] -= coef[j] * w * np.sign(diff)
        dO[b] += coef[j] * (1.0 - M.alpha) * outside
        G.add_row("E", int(cand[j]), coef[j] * w * np.sign(diff))
    for b in range(len(branches)):
        backward(tapes[b], dC[b], dO[b], M, G)
    return loss, s


def batch_loss_and_grads(batch, negs, M, want_grads=True, track_sq=False):
    G = Grads(M.P, track_sq) if want_grads else None
    total, scores = 0.0, []
    for i in range(batch.B):
        l, s = query_step(batch.query_nodes(i), int(batch.pos[i]), negs[i], M, batch.B, G)
        total += l
        scores.append(s)
    return total, G, scores


def adam_step(P, state, G, t, hp):
    kw = dict(lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["eps"])
    for name, g in G.dense.items():
        m, v = state[name]
        P[name], state[name][0], state[name][1] = adam_update(P[name], m, v, g, t, **kw)
    for table in TABLES:
        m, v = state[table]
        for i, g in G.rows[table].items():
            P[table][i], m[i], v[i] = adam_update(P[table][i], m[i], v[i], g, t, **kw)


def train_step(batch, negs, params, state, t, hp, track_sq=False):
    """One full step.  params/state are fp64 dicts updated in place; returns (loss, grads)."""
    M = BoxModel(params, hp["gamma"], hp["alpha"])
    M.P = params
    loss, G, _ = batch_loss_and_grads(batch, negs, M, track_sq=track_sq)
    adam_step(params, state, G, t, hp)
    return loss, G
