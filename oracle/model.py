"""Per-query, node-by-node reference of one NGDB training step (numpy, fp64).

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

What is computed (paper sections in brackets):

* A query is a tree of atomic operators -- projection, intersection, negation,
  union -- over anchor entities [Sec. 3.1; Sec. 4.1 "Graph Decomposition"].
  The paper's method batches same-type operators across queries, which is a
  re-ordering of the work and not a change of the result [Sec. 4.1 "Batched
  Execution", Eq. Y = Kernel(X; theta)].  The oracle therefore evaluates every
  query on its own, one node after the other, with the shared parameters of
  each operator type.
* The objective is a sum over queries of a term for the positive answer and
  one for every negative sample [Sec. 4.2 "Vectorized Logit Formulation"],
  with psi = log-sigmoid of a margin minus a distance.
* One optimiser step after all gradients are in [Alg. 1, last line; Adam with
  lr 1e-4 in the hyper-parameter table].

The paper gives no operator formulas; the workload definition does and it is
followed here:
    projection    y = W2 relu(W1 (x + R[r]) + b1) + b2
    negation      y = V2 relu(V1 x + c1) + c2
    intersection  a_k = U2 relu(U1 x_k + u1) + u2 ; w = softmax over k (per
                  coordinate) ; y = sum_k w_k * x_k
    union         disjunctive normal form: the query splits into conjunctive
                  branches; a candidate's score is the max over branches
    score         s(q, e) = gamma - min_b || y_b - Ef[e] ||_1
    loss          L = 1/(2B) sum_i [ -log sigmoid(s(q_i, pos_i))
                                     - 1/K sum_j log sigmoid(-s(q_i, neg_ij)) ]
    entity row    Ef[e] = E[e]                      (no text features)
                  Ef[e] = E[e] + bf16(Wp) Hsem[e]   (frozen bf16 text features)
Kinks: relu'(0) = 0, sign(0) = 0, equal branch distances -> lowest branch.
Adam: textbook, beta = (0.9, 0.999), eps 1e-8, no weight decay; dense on the
MLP weights (and Wp); on the embedding tables E and R only rows that received
a contribution in this step are updated (lazy / row-sparse Adam), with the
global step count in the bias correction.
"""
import numpy as np

OP_ANCHOR, OP_PROJ, OP_INTER, OP_NEG, OP_UNION = 0, 1, 2, 3, 4


class Unsupported(Exception):
    """Union below an intersection or a negation, or a query that is a bare anchor."""


# ----------------------------------------------------------------------------
# small helpers
# ----------------------------------------------------------------------------
def softplus(x):
    """log(1 + exp(x)) without overflow."""
    x = np.asarray(x, np.float64)
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def sigmoid(x):
    x = np.asarray(x, np.float64)
    e = np.exp(-np.abs(x))
    return np.where(x >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def bf16_round(x):
    """Round fp32 values to the nearest bf16 (ties to even); returned as fp64."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & np.uint32(0xFFFF0000)
    return b.view(np.float32).astype(np.float64)


def bf16_bits_to_f64(bits):
    return (np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(params):
    return {k: np.asarray(v, np.float64) for k, v in params.items()}


# ----------------------------------------------------------------------------
# queries
# ----------------------------------------------------------------------------
def query_tree(nodes):
    """Nested tuple for one query given as [(op, arg, [input positions])], root last."""
    def build(j):
        op, arg, ins = nodes[j]
        if op == OP_ANCHOR:
            return ("e", arg)
        if op == OP_PROJ:
            return ("p", arg, build(ins[0]))
        if op == OP_NEG:
            return ("n", build(ins[0]))
        if op == OP_INTER:
            return ("i",) + tuple(build(k) for k in ins)
        if op == OP_UNION:
            return ("u",) + tuple(build(k) for k in ins)
        raise ValueError(op)
    return build(len(nodes) - 1)


def dnf(tree):
    """Conjunctive branches of a query (disjunctive normal form), in input order.

    A union may sit at the root or under projections only; the projections
    above it are repeated in every branch.
    """
    kind = tree[0]
    if kind == "e":
        return [tree]
    if kind == "p":
        return [("p", tree[1], b) for b in dnf(tree[2])]
    if kind == "u":
        out = []
        for c in tree[1:]:
            out.extend(dnf(c))
        return out
    kids = []
    for c in tree[1:]:
        b = dnf(c)
        if len(b) != 1:
            raise Unsupported("union below an intersection or negation")
        kids.append(b[0])
    return [(kind,) + tuple(kids)]


# ----------------------------------------------------------------------------
# model
# ----------------------------------------------------------------------------
class Model:
    """Parameters in fp64 plus the entity-row rule Ef[e]."""

    def __init__(self, params, gamma, sem_bits=None, score_bf16=False):
        self.P = to_f64(params)
        self.gamma = float(gamma)
        # candidate rows (positives, negatives, ranking) read from a bf16 copy of E; anchors and
        # the optimiser keep the fp32 rows; a rounded row passes its gradient on unchanged
        self.score_bf16 = bool(score_bf16)
        self.sem_bits = sem_bits                 # [N, d_sem] uint16 bf16 patterns or None
        self.Wp_used = bf16_round(params["Wp"]) if sem_bits is not None else None

    def sem(self, e):
        return bf16_bits_to_f64(self.sem_bits[e])

    def entity(self, e):
        """Ef[e] for an id or an array of ids."""
        row = self.P["E"][e]
        if self.sem_bits is not None:
            row = row + self.sem(e) @ self.Wp_used.T
        return row

    def candidate(self, e):
        """The row of entity e as the scoring and ranking passes read it."""
        return bf16_round(self.P["E"][e]) if self.score_bf16 else self.entity(e)


def mlp_forward(x, Wa, ba, Wb, bb):
    pre = Wa @ x + ba
    hid = np.maximum(pre, 0.0)
    return Wb @ hid + bb, (x, pre, hid)


def mlp_backward(dy, tape, Wa, Wb):
    """Returns dx and the four parameter gradients of y = Wb relu(Wa x + ba) + bb."""
    x, pre, hid = tape
    dWb = np.outer(dy, hid)
    dbb = dy
    dhid = Wb.T @ dy
    dpre = dhid * (pre > 0.0)
    dWa = np.outer(dpre, x)
    dba = dpre
    dx = Wa.T @ dpre
    return dx, dWa, dba, dWb, dbb


def forward(tree, M):
    """Embedding of a conjunctive (union-free) tree and what backward needs."""
    P = M.P
    kind = tree[0]
    if kind == "e":
        return M.entity(tree[1]), ("e", tree[1])
    if kind == "p":
        x, tx = forward(tree[2], M)
        y, t = mlp_forward(x + P["R"][tree[1]], P["W1"], P["b1"], P["W2"], P["b2"])
        return y, ("p", tree[1], tx, t)
    if kind == "n":
        x, tx = forward(tree[1], M)
        y, t = mlp_forward(x, P["V1"], P["c1"], P["V2"], P["c2"])
        return y, ("n", tx, t)
    if kind == "i":
        xs, txs, tapes, att = [], [], [], []
        for c in tree[1:]:
            x, tx = forward(c, M)
            a, t = mlp_forward(x, P["U1"], P["u1"], P["U2"], P["u2"])
            xs.append(x)
            txs.append(tx)
            tapes.append(t)
            att.append(a)
        X = np.stack(xs)                       # [k, d]
        A = np.stack(att)
        A = A - A.max(axis=0, keepdims=True)
        Wt = np.exp(A)
        Wt /= Wt.sum(axis=0, keepdims=True)    # softmax over the k inputs, per coordinate
        return (Wt * X).sum(axis=0), ("i", txs, tapes, X, Wt)
    raise Unsupported("forward() takes conjunctive trees; split unions with dnf()")


class Grads:
    """Gradient accumulators.  Table gradients are kept per touched row; `mass` keeps, per row,
    the sum of the largest entries of its contributions (contributions of opposite sign cancel;
    the accuracy a sum of fp32 terms can have is set by the terms, not by what is left of them)."""

    def __init__(self, P, track_sq=False):
        self.dense = {k: np.zeros_like(v) for k, v in P.items() if k not in ("E", "R")}
        # optional, for tests: per element the sum of the squared contributions (the square root is
        # the scale on which independent rounding errors of the contributions add up)
        self.dense_sq = {k: np.zeros_like(v) for k, v in self.dense.items()} if track_sq else None
        self.rows = {"E": {}, "R": {}}
        self.mass = {"E": {}, "R": {}}

    def add(self, name, val):
        self.dense[name] += val
        if self.dense_sq is not None:
            self.dense_sq[name] += np.square(val)

    def add_row(self, table, idx, vec):
        r = self.rows[table]
        idx = int(idx)
        if idx in r:
            r[idx] = r[idx] + vec
        else:
            r[idx] = np.array(vec, np.float64)
        self.mass[table][idx] = self.mass[table].get(idx, 0.0) + float(np.abs(vec).max())

    def table_dense(self, table, shape):
        out = np.zeros(shape, np.float64)
        for i, v in self.rows[table].items():
            out[i] = v
        return out


def entity_backward(e, g, M, G):
    """Back-propagate g = dL/dEf[e] to the structural row and the text projection."""
    G.add_row("E", e, g)
    if M.sem_bits is not None:
        G.add("Wp", np.outer(g, M.sem(e)))


def backward(tape, dy, M, G):
    P = M.P
    kind = tape[0]
    if kind == "e":
        entity_backward(tape[1], dy, M, G)
    elif kind == "p":
        _, r, tx, t = tape
        dz, dWa, dba, dWb, dbb = mlp_backward(dy, t, P["W1"], P["W2"])
        G.add("W1", dWa)
        G.add("b1", dba)
        G.add("W2", dWb)
        G.add("b2", dbb)
        G.add_row("R", r, dz)
        backward(tx, dz, M, G)
    elif kind == "n":
        _, tx, t = tape
        dx, dWa, dba, dWb, dbb = mlp_backward(dy, t, P["V1"], P["V2"])
        G.add("V1", dWa)
        G.add("c1", dba)
        G.add("V2", dWb)
        G.add("c2", dbb)
        backward(tx, dx, M, G)
    elif kind == "i":
        _, txs, tapes, X, Wt = tape
        # y = sum_k w_k x_k with w = softmax(a):  dy/dx_k (direct) = w_k,
        # dy/da_k = w_k (x_k - y)
        t_all = (Wt * X * dy).sum(axis=0)
        for k in range(X.shape[0]):
            da = Wt[k] * (dy * X[k] - t_all)
            dxa, dWa, dba, dWb, dbb = mlp_backward(da, tapes[k], P["U1"], P["U2"])
            G.add("U1", dWa)
            G.add("u1", dba)
            G.add("U2", dWb)
            G.add("u2", dbb)
            backward(txs[k], Wt[k] * dy + dxa, M, G)
    else:
        raise ValueError(kind)


def score(Y, e_rows, gamma):
    """s = gamma - min_b ||y_b - e||_1 for branch embeddings Y [nb, d] and rows [m, d].

    Returns (scores [m], winning branch [m]); ties go to the lowest branch.
    """
    dist = np.abs(Y[:, None, :] - e_rows[None, :, :]).sum(axis=2)     # [nb, m]
    win = np.argmin(dist, axis=0)
    return gamma - dist[win, np.arange(dist.shape[1])], win


def pair_loss_terms(s_pos, s_neg):
    """-log sigmoid(s+) - mean_j log sigmoid(-s-_j) for one query."""
    return float(softplus(-s_pos)) + float(np.mean(softplus(s_neg)))


def query_step(nodes, pos, negs, M, B, G=None):
    """Loss contribution of one query (already divided by 2B) and, if G is
    given, its gradient contributions."""
    branches = dnf(query_tree(nodes))
    if any(b[0] == "e" for b in branches):
        raise Unsupported("a query must contain at least one operator")
    Ys, tapes = [], []
    for b in branches:
        y, t = forward(b, M)
        Ys.append(y)
        tapes.append(t)
    Y = np.stack(Ys)
    cand = np.concatenate([[pos], np.asarray(negs, np.int64)])
    rows = M.candidate(cand)
    s, win = score(Y, rows, M.gamma)
    K = len(cand) - 1
    loss = pair_loss_terms(s[0], s[1:]) / (2.0 * B)
    if G is None:
        return loss, s
    # dL/ds: positive -sigmoid(-s)/(2B); negatives sigmoid(s)/(2BK)
    c = np.empty_like(s)
    c[0] = -sigmoid(-s[0]) / (2.0 * B)
    c[1:] = sigmoid(s[1:]) / (2.0 * B * K)
    sgn = np.sign(Y[win] - rows)               # [m, d]; ds/dy_win = -sgn, ds/dEf = +sgn
    dY = np.zeros_like(Y)
    for j in range(len(cand)):
        dY[win[j]] -= c[j] * sgn[j]
        entity_backward(int(cand[j]), c[j] * sgn[j], M, G)
    for b in range(len(branches)):
        backward(tapes[b], dY[b], M, G)
    return loss, s


def batch_loss_and_grads(batch, negs, M, want_grads=True, track_sq=False):
    """Sum over the queries of a batch, each handled on its own.

    batch: object with B, pos and query_nodes(i); negs: [B, K] ints.
    Returns (loss, Grads or None, list of per-query score vectors).
    """
    G = Grads(M.P, track_sq) if want_grads else None
    total, scores = 0.0, []
    for i in range(batch.B):
        l, s = query_step(batch.query_nodes(i), int(batch.pos[i]), negs[i], M, batch.B, G)
        total += l
        scores.append(s)
    return total, G, scores


# ----------------------------------------------------------------------------
# optimiser
# ----------------------------------------------------------------------------
def adam_update(p, m, v, g, t, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8):
    """Textbook Adam on arrays of any shape; returns new (p, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return p - lr * mhat / (np.sqrt(vhat) + eps), m, v


def adam_step(P, state, G, t, hp):
    """In-place Adam step t (1-based) on fp64 parameters P with state {name: (m, v)}.

    Dense tensors: every element.  E and R: only rows present in G.rows.
    """
    kw = dict(lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["eps"])
    for name, g in G.dense.items():
        m, v = state[name]
        P[name], state[name][0], state[name][1] = adam_update(P[name], m, v, g, t, **kw)
    for table in ("E", "R"):
        m, v = state[table]
        for i, g in G.rows[table].items():
            P[table][i], m[i], v[i] = adam_update(P[table][i], m[i], v[i], g, t, **kw)


def new_state(P):
    return {k: [np.zeros_like(v), np.zeros_like(v)] for k, v in P.items()}


def train_step(batch, negs, params, state, t, hp, sem_bits=None, track_sq=False, score_bf16=False):
    """One full step.  params/state are fp64 dicts updated in place; returns the loss."""
    M = Model(params, hp["gamma"], sem_bits, score_bf16)
    M.P = params                                   # update the caller's arrays
    loss, G, _ = batch_loss_and_grads(batch, negs, M, track_sq=track_sq)
    adam_step(params, state, G, t, hp)
    return loss, G
