"""Seeded query batches: template trees instantiated by backward random walks.

A query is stored flat (the layout the C boundary takes): per query a run of
nodes in an order where inputs precede their consumer and the root is last.
Node kinds: 0 anchor entity, 1 projection (carries a relation id),
2 intersection, 3 negation, 4 union.
"""
from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

from .configs import TEMPLATES
from .kg import KG

OP_ANCHOR, OP_PROJ, OP_INTER, OP_NEG, OP_UNION = 0, 1, 2, 3, 4
_OPCODE = {"e": OP_ANCHOR, "p": OP_PROJ, "i": OP_INTER, "n": OP_NEG, "u": OP_UNION}


@dataclass
class QueryBatch:
    B: int
    node_off: np.ndarray   # [B+1] int32
    op: np.ndarray         # [n_nodes] uint8
    arg: np.ndarray        # [n_nodes] int32  entity id (anchor) / relation id (projection) / 0
    in_off: np.ndarray     # [n_nodes+1] int32
    in_idx: np.ndarray     # [n_inputs] int32  indices local to the query
    pos: np.ndarray        # [B] int32  positive answer entity
    names: List[str]       # template name per query ("" if built from explicit trees)

    def query_nodes(self, i: int):
        """Nodes of query i as a list of (op, arg, [local input indices])."""
        out = []
        for n in range(int(self.node_off[i]), int(self.node_off[i + 1])):
            ins = self.in_idx[int(self.in_off[n]):int(self.in_off[n + 1])]
            out.append((int(self.op[n]), int(self.arg[n]), [int(x) for x in ins]))
        return out

    def select(self, idx: Sequence[int]) -> "QueryBatch":
        """Sub-batch made of the listed queries, in the listed order."""
        trees = [self.tree(i) for i in idx]
        qb = batch_from_trees(trees, [int(self.pos[i]) for i in idx])
        qb.names = [self.names[i] for i in idx]
        return qb

    def tree(self, i: int):
        """Query i as a nested tuple: ('e', ent) / ('p', rel, x) / ('i', x..) / ('n', x) / ('u', x..)."""
        nodes = self.query_nodes(i)

        def build(j):
            op, arg, ins = nodes[j]
            if op == OP_ANCHOR:
                return ("e", arg)
            if op == OP_PROJ:
                return ("p", arg, build(ins[0]))
            if op == OP_NEG:
                return ("n", build(ins[0]))
            return ("i" if op == OP_INTER else "u",) + tuple(build(k) for k in ins)

        return build(len(nodes) - 1)


def batch_from_trees(trees, pos) -> QueryBatch:
    """Flatten nested-tuple queries (post-order, root last) into a QueryBatch."""
    node_off, op, arg, in_off, in_idx = [0], [], [], [0], []
    for tree in trees:
        base = len(op)

        def emit(t):
            kind = t[0]
            if kind == "e":
                ins, a = [], t[1]
            elif kind == "p":
                ins, a = [emit(t[2])], t[1]
            elif kind == "n":
                ins, a = [emit(t[1])], 0
            else:
                ins, a = [emit(c) for c in t[1:]], 0
            op.append(_OPCODE[kind])
            arg.append(a)
            in_idx.extend(ins)
            in_off.append(len(in_idx))
            return len(op) - 1 - base

        emit(tree)
        node_off.append(len(op))
    return QueryBatch(
        B=len(trees),
        node_off=np.asarray(node_off, np.int32),
        op=np.asarray(op, np.uint8),
        arg=np.asarray(arg, np.int32),
        in_off=np.asarray(in_off, np.int32),
        in_idx=np.asarray(in_idx, np.int32),
        pos=np.asarray(pos, np.int32),
        names=[""] * len(trees),
    )


class _Retry(Exception):
    pass


def _instantiate(tmpl, v: int, kg: KG, rng, answer=None):
    """Instantiate template `tmpl` so that entity v is (one of) its answers."""
    kind = tmpl[0]
    if kind == "e":
        return ("e", int(v))
    if kind == "p":
        lo, hi = int(kg.in_off[v]), int(kg.in_off[v + 1])
        if hi == lo:
            raise _Retry
        j = lo + int(rng.integers(0, hi - lo))
        u, r = int(kg.head[j]), int(kg.rel[j])
        if answer is not None and tmpl[1][0] == "e" and kg.has_triple(u, r, answer):
            raise _Retry          # a one-hop negated branch must not contain the answer
        return ("p", r, _instantiate(tmpl[1], u, kg, rng))
    if kind == "n":
        other = int(kg.tail[int(rng.integers(0, kg.T))])
        return ("n", _instantiate(tmpl[1], other, kg, rng, answer=v))
    if kind == "i":
        kids = []
        for c in tmpl[1:]:
            for _ in range(8):
                k = _instantiate(c, v, kg, rng)
                if k not in kids:
                    break
            else:
                raise _Retry
            kids.append(k)
        return ("i",) + tuple(kids)
    if kind == "u":
        first = _instantiate(tmpl[1], v, kg, rng)
        rest = [_instantiate(c, int(kg.tail[int(rng.integers(0, kg.T))]), kg, rng)
                for c in tmpl[2:]]
        return ("u", first) + tuple(rest)
    raise ValueError(kind)


def make_batch(kg: KG, B: int, mix: dict, seed: int) -> QueryBatch:
    """B queries whose templates follow `mix`; the walk's end point is the positive answer."""
    rng = np.random.default_rng(seed)
    names = sorted(mix)
    p = np.asarray([mix[n] for n in names], np.float64)
    p /= p.sum()
    drawn = rng.choice(len(names), size=B, p=p)
    trees, pos, used = [], [], []
    for b in range(B):
        name = names[int(drawn[b])]
        for _ in range(1000):
            t = int(kg.tail[int(rng.integers(0, kg.T))])
            try:
                tree = _instantiate(TEMPLATES[name], t, kg, rng)
            except _Retry:
                continue
            break
        else:
            raise RuntimeError("query instantiation kept failing for " + name)
        trees.append(tree)
        pos.append(t)
        used.append(name)
    qb = batch_from_trees(trees, pos)
    qb.names = used
    return qb


def make_negatives(N: int, B: int, K: int, seed: int) -> np.ndarray:
    """[B, K] int32 negatives, i.i.d. uniform over the entities (with replacement, unfiltered)."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, N, size=(B, K), dtype=np.int32)
