"""ctypes binding of libngdb.so: argument marshalling only.

Every step of the training path runs inside the library's HIP kernels; this
module converts numpy / torch objects to the plain pointers of include/ngdb.h
and back.  PyTorch is used for device memory and streams.  If the library is
missing the import fails loudly -- there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libngdb.so")

MLP_NAMES = ("W1", "b1", "W2", "b2", "V1", "c1", "V2", "c2", "U1", "u1", "U2", "u2")
TENSOR_NAMES = ("E", "R") + MLP_NAMES
BOX_TENSOR_NAMES = ("E", "R", "Ro") + MLP_NAMES[4:]      # the box family has no projection MLP
FAMILY_VEC, FAMILY_BOX = 0, 1

NGDB_OK = 0
ERR_ARG, ERR_UNSUPPORTED, ERR_RANGE, ERR_OOM, ERR_HIP, ERR_STATE = -1, -2, -3, -4, -5, -6


class NgdbError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libngdb error %d: %s" % (code, text))
        self.code = code


class Config(C.Structure):
    _fields_ = [("n_entities", C.c_int32), ("n_relations", C.c_int32), ("d", C.c_int32), ("h", C.c_int32),
                ("d_sem", C.c_int32), ("num_streams", C.c_int32), ("gamma", C.c_float), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("schedule", C.c_int32),
                ("b_max", C.c_int32), ("family", C.c_int32), ("box_alpha", C.c_float), ("score_bf16", C.c_int32),
                ("b_max_queries", C.c_int32), ("k_max", C.c_int32), ("max_nodes_per_query", C.c_int32)]


class Tensor(C.Structure):
    _fields_ = [("p", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p)]


class Params(C.Structure):
    _fields_ = [(n, Tensor) for n in TENSOR_NAMES] + [("Wp", Tensor), ("H_sem", C.c_void_p), ("step", C.c_int64),
                                                       ("Ro", Tensor)]


class QueryBatchC(C.Structure):
    _fields_ = [("n_queries", C.c_int32), ("node_off", C.c_void_p), ("op", C.c_void_p), ("arg", C.c_void_p),
                ("in_off", C.c_void_p), ("in_idx", C.c_void_p), ("pos", C.c_void_p)]


_PLAN_COUNTS = ("n_queries", "n_groups", "n_levels", "n_slots", "n_anchor", "n_proj", "n_inter", "n_neg",
                "n_int_rows", "n_roots", "n_refs", "n_r_uniq", "peak_live")
SCHED_LEVEL, SCHED_MAX_FILL = 0, 1
_PLAN_ARRAYS = ("lvl_off", "g_level", "g_type", "g_nin", "g_n", "g_out_base", "g_mlp_base", "g_ref_off",
                "g_rel_off", "in_ref", "in_gslot", "rel", "root_off", "root_slot", "anchor_ent", "pos",
                "r_uniq", "r_seg_off", "r_src")


class PlanView(C.Structure):
    _fields_ = ([(n, C.c_int32) for n in _PLAN_COUNTS] + [(n, C.POINTER(C.c_int32)) for n in _PLAN_ARRAYS] +
                [("n_f_rows", C.c_int32), ("f_step_rows", C.c_int32 * 3), ("f_row", C.POINTER(C.c_int32))])


class GradView(C.Structure):
    _fields_ = [("n_e_uniq", C.c_int32), ("n_e_contrib", C.c_int32), ("n_r_uniq", C.c_int32),
                ("n_slots", C.c_int32), ("n_pairs", C.c_int32),
                ("e_uniq", C.c_void_p), ("e_seg_off", C.c_void_p), ("e_src", C.c_void_p),
                ("gE", C.c_void_p), ("gR", C.c_void_p), ("g_mlp", C.c_void_p * 12), ("g_Wp", C.c_void_p),
                ("act", C.c_void_p), ("dact", C.c_void_p), ("n_grad_rows", C.c_int32),
                ("pair_score", C.c_void_p), ("loss_terms", C.c_void_p),
                ("gRo", C.c_void_p), ("off", C.c_void_p), ("doff", C.c_void_p), ("e_shadow", C.c_void_p)]


TIMING_CLASSES = ("index", "sem", "gemm_fwd", "inter", "score", "gemm_bwd", "wgrad", "table_E", "table_R",
                  "adam")


class Timing(C.Structure):
    _fields_ = [("ms", C.c_double * 10), ("brackets", C.c_int64 * 10), ("route_ms", (C.c_double * 2) * 10),
                ("route_launches", (C.c_int64 * 2) * 10), ("route_flop", (C.c_double * 2) * 10)]


def load_library(path=LIB_PATH):
    if not os.path.exists(path):
        raise ImportError("libngdb.so has not been built (run `python -m paper_2602_21597_amd.build`): " + path)
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    sig = {
        "ngdb_create": (C.c_int, [C.POINTER(Config), C.POINTER(vp)]),
        "ngdb_destroy": (None, [vp]),
        "ngdb_bind_params": (C.c_int, [vp, C.POINTER(Params)]),
        "ngdb_plan": (C.c_int, [vp, C.POINTER(QueryBatchC), C.POINTER(vp)]),
        "ngdb_plan_host": (C.c_int, [i32, i32, C.POINTER(QueryBatchC), C.POINTER(vp)]),
        "ngdb_plan_host_sched": (C.c_int, [i32, i32, C.POINTER(QueryBatchC), i32, i32, C.POINTER(vp)]),
        "ngdb_plan_export": (C.c_int, [vp, C.POINTER(PlanView)]),
        "ngdb_plan_free": (None, [vp]),
        "ngdb_train_step": (C.c_int, [vp, vp, vp, i32, vp, vp]),
        "ngdb_forward_backward": (C.c_int, [vp, vp, vp, i32, vp, vp]),
        "ngdb_get_grads": (C.c_int, [vp, C.POINTER(GradView)]),
        "ngdb_score": (C.c_int, [vp, vp, vp, i32, i32, vp, vp, vp, vp]),
        "ngdb_score_noalloc": (C.c_int, [vp, vp, vp, i32, vp, vp]),
        "ngdb_score_noalloc_bytes": (C.c_size_t, [vp, vp]),
        "ngdb_rank_answers": (C.c_int, [vp, vp, vp, vp, i32, vp, vp, vp]),
        "ngdb_rank_metrics": (C.c_int, [vp, vp, vp, i32, vp, vp]),
        "ngdb_sampler_create": (C.c_int, [i32, i32, i64, vp, vp, vp, C.c_char_p, vp, C.c_uint64, i32, C.POINTER(vp)]),
        "ngdb_sampler_next": (C.c_int, [vp, i32, i32, C.POINTER(QueryBatchC), C.POINTER(vp), C.POINTER(vp)]),
        "ngdb_sampler_destroy": (None, [vp]),
        "ngdb_sampler_last_error": (C.c_char_p, [vp]),
        "ngdb_debug_mlp": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, C.POINTER(C.c_int32), vp]),
        "ngdb_debug_gemm": (C.c_int, [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32,
                                      vp, i32, vp]),
        "ngdb_debug_copy": (C.c_int, [vp, vp, C.c_size_t, vp]),
        "ngdb_debug_stream": (C.c_int, [i32, vp, vp, C.c_size_t, vp, i64, i32, vp]),
        "ngdb_set_timing": (C.c_int, [vp, C.c_uint32]),
        "ngdb_get_timing": (C.c_int, [vp, C.POINTER(Timing), C.c_int]),
        "ngdb_copy_to_host": (C.c_int, [vp, vp, C.c_size_t]),
        "ngdb_step_count": (i64, [vp]),
        "ngdb_debug_alloc_count": (i64, [vp]),
        "ngdb_strerror": (C.c_char_p, [C.c_int]),
        "ngdb_last_error": (C.c_char_p, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, np.int32)


class _BatchArrays:
    """Keeps the numpy arrays alive while the C struct points at them."""

    def __init__(self, qb):
        self.keep = [_i32(qb.node_off), np.ascontiguousarray(qb.op, np.uint8), _i32(qb.arg), _i32(qb.in_off),
                     _i32(qb.in_idx), _i32(qb.pos)]
        p = [a.ctypes.data if a.size else None for a in self.keep]
        self.c = QueryBatchC(int(qb.B), p[0], p[1], p[2], p[3], p[4], p[5])


class Plan:
    def __init__(self, handle, owner=None):
        self.handle = handle
        self.owner = owner      # keeps the engine (the plan's context) alive as long as the plan

    def export(self):
        """All plan arrays as a dict of numpy int32 copies / ints."""
        v = PlanView()
        _check(lib().ngdb_plan_export(self.handle, C.byref(v)), None)
        out = {n: int(getattr(v, n)) for n in _PLAN_COUNTS}
        sizes = dict(lvl_off=out["n_levels"] + 2, in_ref=out["n_refs"], in_gslot=out["n_refs"],
                     rel=out["n_proj"], root_off=out["n_queries"] + 1, root_slot=out["n_roots"],
                     anchor_ent=out["n_anchor"], pos=out["n_queries"], r_uniq=out["n_r_uniq"],
                     r_seg_off=out["n_r_uniq"] + 1, r_src=out["n_proj"])
        for n in _PLAN_ARRAYS:
            cnt = sizes.get(n, out["n_groups"])
            p = getattr(v, n)
            out[n] = np.ctypeslib.as_array(p, shape=(cnt,)).copy() if cnt else np.zeros(0, np.int32)
        out["n_f_rows"] = int(v.n_f_rows)
        out["f_step_rows"] = np.asarray(list(v.f_step_rows), np.int32)
        out["f_row"] = (np.ctypeslib.as_array(v.f_row, shape=(out["n_slots"],)).copy() if out["n_slots"]
                        else np.zeros(0, np.int32))
        return out

    def free(self):
        if self.handle:
            lib().ngdb_plan_free(self.handle)
            self.handle = None
        self.owner = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _check(rc, ctx):
    if rc != NGDB_OK:
        L = lib()
        text = L.ngdb_strerror(rc).decode()
        if ctx:
            detail = L.ngdb_last_error(ctx).decode()
            if detail:
                text += " (" + detail + ")"
        raise NgdbError(rc, text)


def plan_host(n_entities, n_relations, qb, schedule=SCHED_LEVEL, b_max=0):
    """Host-only planning (no device needed); the plan can be exported, not executed."""
    arrs = None if isinstance(qb, QueryBatchC) else _BatchArrays(qb)    # keeps the numpy arrays alive
    c = qb if arrs is None else arrs.c
    h = C.c_void_p()
    _check(lib().ngdb_plan_host_sched(int(n_entities), int(n_relations), C.byref(c), int(schedule), int(b_max),
                                      C.byref(h)), None)
    return Plan(h)


def copy_to_host(dev_ptr, shape, dtype):
    out = np.empty(shape, dtype)
    if out.size:
        _check(lib().ngdb_copy_to_host(out.ctypes.data, dev_ptr, out.nbytes), None)
    return out


def debug_gemm(A, B, M, N, K, a_kcontig=True, b_kcontig=True, bias=None, relu=False, mask=None, addend=None,
               dst_row=None, out_rows=None, arith=0):
    """Runs the library's contraction kernel on torch device tensors; returns C [out_rows or M, N]."""
    import torch
    Cm = torch.zeros((out_rows or M, N), dtype=torch.float32, device=A.device)
    p = lambda t: t.data_ptr() if t is not None else None
    ld = lambda t: int(t.stride(0)) if t is not None else 0
    _check(lib().ngdb_debug_gemm(p(A), p(B), p(Cm), M, N, K, ld(A), ld(B), ld(Cm), int(a_kcontig), int(b_kcontig),
                                 p(bias), int(relu), p(mask), ld(mask), p(addend), ld(addend), p(dst_row), int(arith),
                                 C.c_void_p(torch.cuda.current_stream().cuda_stream)), None)
    torch.cuda.synchronize()
    return Cm


def debug_mlp(X, W1, b1, W2, b2, mask=None, backward=False):
    """The two chained launches of one operator MLP with operands as bf16 pieces (ngdb_debug_mlp) on
    torch device tensors; returns (H, Y, used)."""
    import torch
    M, d = X.shape
    h = W1.shape[0]
    H = torch.zeros((M, h), dtype=torch.float32, device=X.device)
    Y = torch.zeros((M, d), dtype=torch.float32, device=X.device)
    used = C.c_int32(0)
    p = lambda t: t.data_ptr() if t is not None else None
    _check(lib().ngdb_debug_mlp(p(X), p(W1), p(b1), p(W2), p(b2), p(mask), p(H), p(Y), M, d, h, int(backward),
                                C.byref(used), C.c_void_p(torch.cuda.current_stream().cuda_stream)), None)
    return H, Y, used.value


def debug_copy(dst, src):
    """Plain copy kernel between two equally sized torch device tensors (bytes multiple of 16)."""
    import torch
    nbytes = src.numel() * src.element_size()
    _check(lib().ngdb_debug_copy(dst.data_ptr(), src.data_ptr(), nbytes,
                                 C.c_void_p(torch.cuda.current_stream().cuda_stream)), None)
    return nbytes


STREAM_COPY, STREAM_READ, STREAM_WRITE, STREAM_GATHER, STREAM_UPDATE, STREAM_COPY_NT, STREAM_UPDATE_NT = range(7)


def debug_stream(mode, dst, src=None, rows=None, row_floats=0, nbytes=None):
    """One launch of a calibration access pattern (ngdb_debug_stream) on torch device tensors."""
    import torch
    if nbytes is None:
        ref = src if mode in (STREAM_COPY, STREAM_READ, STREAM_COPY_NT) else dst
        nbytes = ref.numel() * ref.element_size()
    _check(lib().ngdb_debug_stream(int(mode), dst.data_ptr(), src.data_ptr() if src is not None else None, int(nbytes),
                                   rows.data_ptr() if rows is not None else None,
                                   int(rows.numel()) if rows is not None else 0, int(row_floats),
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream)), None)
    return nbytes


class SampledBatch:
    """A batch the sampler produced, copied out of its buffers: the flat query arrays of the
    C boundary (same attribute names as workloads.QueryBatch), negatives and template ids."""

    def __init__(self, c, neg_ptr, tmpl_ptr, K, names):
        B = int(c.n_queries)
        take = lambda ptr, n, dt: (np.ctypeslib.as_array(C.cast(ptr, C.POINTER(dt)), shape=(n,)).copy() if n
                                   else np.zeros(0, dt))
        self.B = B
        self.node_off = take(c.node_off, B + 1, C.c_int32)
        n_nodes = int(self.node_off[-1]) if B else 0
        self.op = take(c.op, n_nodes, C.c_uint8)
        self.arg = take(c.arg, n_nodes, C.c_int32)
        self.in_off = take(c.in_off, n_nodes + 1, C.c_int32)
        self.in_idx = take(c.in_idx, int(self.in_off[-1]), C.c_int32)
        self.pos = take(c.pos, B, C.c_int32)
        self.negs = take(neg_ptr, B * K, C.c_int32).reshape(B, K)
        self.names = [names[int(t)] for t in take(tmpl_ptr, B, C.c_uint8)]

    def query_nodes(self, i):
        """Nodes of query i as a list of (op, arg, [local input indices]), root last."""
        out = []
        for n in range(int(self.node_off[i]), int(self.node_off[i + 1])):
            ins = self.in_idx[int(self.in_off[n]):int(self.in_off[n + 1])]
            out.append((int(self.op[n]), int(self.arg[n]), [int(x) for x in ins]))
        return out


class Sampler:
    """Online query sampler over a graph given as triple arrays (host, no device needed)."""

    def __init__(self, n_entities, n_relations, head, rel, tail, templates, weights=None, seed=0, n_threads=4):
        self.names = list(templates)
        self._keep = [_i32(head), _i32(rel), _i32(tail)]
        w = np.ascontiguousarray(weights, np.float32) if weights is not None else None
        self.handle = C.c_void_p()
        _check(lib().ngdb_sampler_create(int(n_entities), int(n_relations), int(self._keep[0].shape[0]),
                                         self._keep[0].ctypes.data, self._keep[1].ctypes.data,
                                         self._keep[2].ctypes.data, ",".join(self.names).encode(),
                                         w.ctypes.data if w is not None else None, int(seed), int(n_threads),
                                         C.byref(self.handle)), None)

    def _next(self, n_queries, K):
        c = QueryBatchC()
        neg, tmpl = C.c_void_p(), C.c_void_p()
        rc = lib().ngdb_sampler_next(self.handle, int(n_queries), int(K), C.byref(c), C.byref(neg), C.byref(tmpl))
        if rc != NGDB_OK:
            raise NgdbError(rc, lib().ngdb_strerror(rc).decode() + " (" +
                            lib().ngdb_sampler_last_error(self.handle).decode() + ")")
        return c, neg, tmpl

    def next(self, n_queries, K):
        """A fresh batch copied into numpy arrays (inspection, tests)."""
        c, neg, tmpl = self._next(n_queries, K)
        return SampledBatch(c, neg, tmpl, int(K), self.names)

    def next_raw(self, n_queries, K):
        """A fresh batch left in the sampler's buffers: (the C struct, to be passed to Engine.plan
        as it is; a numpy view [n_queries, K] of the negatives).  Both are valid until the call
        after the next one on this sampler."""
        c, neg, _ = self._next(n_queries, K)
        n = int(n_queries) * int(K)
        negs = (np.ctypeslib.as_array(C.cast(neg, C.POINTER(C.c_int32)), shape=(n,)).reshape(int(n_queries), int(K))
                if n else np.zeros((int(n_queries), int(K)), np.int32))
        return c, negs

    def close(self):
        if self.handle:
            lib().ngdb_sampler_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Engine:
    """One libngdb context plus the device tensors bound to it."""

    def __init__(self, n_entities, n_relations, d, h, gamma, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8,
                 d_sem=0, num_streams=1, device="cuda:0", schedule=SCHED_LEVEL, b_max=0, family=FAMILY_VEC,
                 box_alpha=0.02, score_bf16=False, b_max_queries=0, k_max=0, max_nodes_per_query=0):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("libngdb needs a GPU; there is no CPU path")
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = Config(n_entities, n_relations, d, h, d_sem, num_streams, gamma, lr, beta1, beta2, eps,
                          int(schedule), int(b_max), int(family), float(box_alpha), int(bool(score_bf16)),
                          int(b_max_queries), int(k_max), int(max_nodes_per_query))
        self.ctx = C.c_void_p()
        _check(lib().ngdb_create(C.byref(self.cfg), C.byref(self.ctx)), None)
        self.tensors = {}
        self._loss = torch.zeros(1, dtype=torch.float32, device=self.device)

    # ---- parameters
    def tensor_names(self):
        if self.cfg.family == FAMILY_BOX:
            return BOX_TENSOR_NAMES
        return TENSOR_NAMES + (("Wp",) if self.cfg.d_sem else ())

    def bind_numpy(self, params, step=0, sem_bits=None):
        """Uploads fp32 numpy parameters, creates zero moments, binds them.  With text features
        (d_sem > 0) params holds "Wp" and sem_bits is the [N, d_sem] uint16 array of bf16 patterns."""
        t = self.torch
        self.tensors = {}
        for name in self.tensor_names():
            p = t.from_numpy(np.ascontiguousarray(params[name], np.float32)).to(self.device)
            self.tensors[name] = (p, t.zeros_like(p), t.zeros_like(p))
        self.H_sem = None
        if self.cfg.d_sem:
            assert sem_bits is not None and sem_bits.dtype == np.uint16
            assert sem_bits.shape == (self.cfg.n_entities, self.cfg.d_sem)
            # int16 carries the bit patterns: torch has no uint16 arithmetic, none is needed
            self.H_sem = t.from_numpy(np.ascontiguousarray(sem_bits).view(np.int16)).to(self.device)
        self.bind(step)

    def bind(self, step=0):
        P = Params()
        for name in self.tensor_names():
            p, m, v = self.tensors[name]
            setattr(P, name, Tensor(p.data_ptr(), m.data_ptr(), v.data_ptr()))
        if self.H_sem is not None:
            P.H_sem = self.H_sem.data_ptr()
        P.step = int(step)
        _check(lib().ngdb_bind_params(self.ctx, C.byref(P)), self.ctx)

    def params_numpy(self, which="p"):
        k = "pmv".index(which)
        self.torch.cuda.synchronize()
        return {n: ts[k].cpu().numpy() for n, ts in self.tensors.items()}

    # ---- planning / steps
    def plan(self, qb):
        """qb: an object with the flat query arrays (workloads.QueryBatch, SampledBatch) or the C
        struct a sampler filled (Sampler.next_raw)."""
        arrs = None if isinstance(qb, QueryBatchC) else _BatchArrays(qb)    # keeps the numpy arrays alive
        c = qb if arrs is None else arrs.c
        h = C.c_void_p()
        _check(lib().ngdb_plan(self.ctx, C.byref(c), C.byref(h)), self.ctx)
        return Plan(h, self)

    def _stream(self, stream):
        return C.c_void_p(stream.cuda_stream if stream is not None else
                          self.torch.cuda.current_stream(self.device).cuda_stream)

    def _neg(self, neg):
        assert neg.dtype == self.torch.int32 and neg.is_cuda and neg.is_contiguous() and neg.dim() == 2
        return neg.data_ptr(), int(neg.shape[1])

    def train_step(self, plan, neg, stream=None, loss_out=None):
        """neg: [B, K] int32 device tensor.  Returns the device tensor that receives the loss."""
        loss = self._loss if loss_out is None else loss_out
        ptr, K = self._neg(neg)
        _check(lib().ngdb_train_step(self.ctx, plan.handle, ptr, K, self._stream(stream), loss.data_ptr()), self.ctx)
        return loss

    def forward_backward(self, plan, neg, stream=None):
        ptr, K = self._neg(neg)
        self._K = K
        _check(lib().ngdb_forward_backward(self.ctx, plan.handle, ptr, K, self._stream(stream),
                                           self._loss.data_ptr()), self.ctx)
        return self._loss

    def grad_view(self):
        """The raw ngdb_grad_view of the last step (device pointers; waits for the device)."""
        gv = GradView()
        _check(lib().ngdb_get_grads(self.ctx, C.byref(gv)), self.ctx)
        return gv

    def read_rows(self, dev_ptr, rows, width, dtype=np.float32):
        """Rows `rows` of a device matrix [*, width] as a numpy copy (one small copy per row)."""
        item = np.dtype(dtype).itemsize
        out = np.empty((len(rows), width), dtype)
        for i, r in enumerate(rows):
            out[i] = copy_to_host(dev_ptr + int(r) * width * item, (width,), dtype)
        return out

    def grads(self):
        """Results of the last forward_backward as numpy copies."""
        gv = GradView()
        _check(lib().ngdb_get_grads(self.ctx, C.byref(gv)), self.ctx)
        d, h = self.cfg.d, self.cfg.h
        U, UR = gv.n_e_uniq, gv.n_r_uniq
        out = dict(
            e_uniq=copy_to_host(gv.e_uniq, (U,), np.int32),
            e_seg_off=copy_to_host(gv.e_seg_off, (U + 1,), np.int32),
            e_src=copy_to_host(gv.e_src, (gv.n_e_contrib,), np.int32),
            act=copy_to_host(gv.act, (gv.n_slots, d), np.float32),
            dact=copy_to_host(gv.dact, (gv.n_grad_rows, d), np.float32),
            pair_score=copy_to_host(gv.pair_score, (gv.n_pairs,), np.float32),
            loss_terms=copy_to_host(gv.loss_terms, (gv.n_pairs // (self._K + 1),), np.float32),
        )
        if gv.gE:
            out["gE"] = copy_to_host(gv.gE, (U, d), np.float32)
            out["gR"] = copy_to_host(gv.gR, (UR, d), np.float32)
        shapes = [(h, d), (h,), (d, h), (d,)] * 3
        for i, name in enumerate(MLP_NAMES):
            if gv.g_mlp[i]:
                out[name] = copy_to_host(gv.g_mlp[i], shapes[i], np.float32)
        if gv.off:
            out["off"] = copy_to_host(gv.off, (gv.n_slots, d), np.float32)
            out["doff"] = copy_to_host(gv.doff, (gv.n_grad_rows, d), np.float32)
        if gv.gRo:
            out["gRo"] = copy_to_host(gv.gRo, (UR, d), np.float32)
        if gv.e_shadow:
            out["e_shadow"] = copy_to_host(gv.e_shadow, (self.cfg.n_entities, d), np.uint16)
        if gv.g_Wp:
            out["Wp"] = copy_to_host(gv.g_Wp, (d, self.cfg.d_sem), np.float32)
        return out

    def score(self, plan, cand, stream=None):
        """cand: [B, C] int32 device tensor -> [B, C] float32 device tensor of scores."""
        t = self.torch
        assert cand.dtype == t.int32 and cand.is_cuda and cand.is_contiguous() and cand.dim() == 2
        out = t.empty(cand.shape, dtype=t.float32, device=self.device)
        _check(lib().ngdb_score(self.ctx, plan.handle, cand.data_ptr(), int(cand.shape[1]), 0, out.data_ptr(),
                                None, None, self._stream(stream)), self.ctx)
        return out

    def score_noalloc(self, plan, cand, out, stream=None):
        """ngdb_score_noalloc: like score(), into the caller's `out` [B, C] float32 device tensor; the
        library allocates nothing (its forward workspace is a static device array)."""
        t = self.torch
        assert cand.dtype == t.int32 and cand.is_cuda and cand.is_contiguous() and cand.dim() == 2
        assert out.dtype == t.float32 and out.is_cuda and out.is_contiguous() and out.shape == cand.shape
        _check(lib().ngdb_score_noalloc(self.ctx, plan.handle, cand.data_ptr(), int(cand.shape[1]), out.data_ptr(),
                                        self._stream(stream)), self.ctx)
        return out

    def score_noalloc_bytes(self, plan):
        return int(lib().ngdb_score_noalloc_bytes(self.ctx, plan.handle))

    def set_timing(self, classes):
        """classes: iterable of names from TIMING_CLASSES (empty = off)."""
        mask = 0
        for n in classes:
            mask |= 1 << TIMING_CLASSES.index(n)
        _check(lib().ngdb_set_timing(self.ctx, mask), self.ctx)

    def get_timing(self, reset=True):
        """{class: (total ms, number of brackets)} since the last reset (waits for the device)."""
        t = Timing()
        _check(lib().ngdb_get_timing(self.ctx, C.byref(t), 1 if reset else 0), self.ctx)
        self.last_routes = {n: {r: (t.route_ms[i][k], int(t.route_launches[i][k]), t.route_flop[i][k])
                                for k, r in enumerate(("fp32", "bf16_split"))}
                            for i, n in enumerate(TIMING_CLASSES)}
        return {n: (t.ms[i], int(t.brackets[i])) for i, n in enumerate(TIMING_CLASSES)}

    def n_touched_entities(self):
        """Number of entity rows touched by the last step (waits for the device)."""
        gv = GradView()
        _check(lib().ngdb_get_grads(self.ctx, C.byref(gv)), self.ctx)
        return int(gv.n_e_uniq)

    def rank_all(self, plan, k, stream=None):
        """All-entity ranking: ([B, k] int32 ids, [B, k] float32 L1 distances), ascending, device tensors."""
        t = self.torch
        B = plan.export()["n_queries"]
        ids = t.empty((B, k), dtype=t.int32, device=self.device)
        dist = t.empty((B, k), dtype=t.float32, device=self.device)
        _check(lib().ngdb_score(self.ctx, plan.handle, None, 0, int(k), None, ids.data_ptr(), dist.data_ptr(),
                                self._stream(stream)), self.ctx)
        return ids, dist

    def rank_answers(self, plan, ans_off, ans, n_take=None, stream=None):
        """Filtered ranks of listed answers.  ans_off [B+1], ans [n_ans]: int32 device tensors;
        n_take [B] int32 device tensor or None.  Returns (ranks [n_ans] int32, distances [n_ans]
        float32, metrics [4] float32 = MRR, Hit@1, Hit@3, Hit@10), device tensors."""
        t = self.torch
        for x in (ans_off, ans):
            assert x.dtype == t.int32 and x.is_cuda and x.is_contiguous() and x.dim() == 1
        n_ans, B = int(ans.shape[0]), int(ans_off.shape[0]) - 1
        ranks = t.empty(max(n_ans, 1), dtype=t.int32, device=self.device)
        dist = t.empty(max(n_ans, 1), dtype=t.float32, device=self.device)
        out = t.empty(4, dtype=t.float32, device=self.device)
        st = self._stream(stream)
        _check(lib().ngdb_rank_answers(self.ctx, plan.handle, ans_off.data_ptr(), ans.data_ptr(), n_ans,
                                       ranks.data_ptr(), dist.data_ptr(), st), self.ctx)
        _check(lib().ngdb_rank_metrics(ranks.data_ptr(), ans_off.data_ptr(),
                                       n_take.data_ptr() if n_take is not None else None, B, out.data_ptr(), st),
               self.ctx)
        return ranks[:n_ans], dist[:n_ans], out

    def alloc_count(self):
        """Device allocations the context has made so far (ngdb_debug_alloc_count)."""
        return int(lib().ngdb_debug_alloc_count(self.ctx))

    def step_count(self):
        return int(lib().ngdb_step_count(self.ctx))

    def close(self):
        if self.ctx:
            lib().ngdb_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
