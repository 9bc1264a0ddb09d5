"""ctypes binding of the C ABI declared in include/marius_hip.h.

Argument marshalling only: every function below forwards to the entry point of the same
name.  torch is used for device memory and the current stream, nothing else.  There is no
fallback: if the shared library is missing the first call raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("MARIUS_HIP_LIB") or os.path.join(_HERE, "libmarius_hip.so")
_lib = None

MODEL_DISTMULT, MODEL_COMPLEX, MODEL_TRANSE, MODEL_DOT = 0, 1, 2, 3
PRECISION_FP32, PRECISION_SPLIT_BF16 = 0, 1
NUM_PHASES = 6
PHASE_NAMES = ("index", "gather", "score_softmax_gq", "neg_grad", "chain_rule", "reduce_adagrad")


class MarError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("marius_hip error %d: %s" % (code, text))
        self.code = code


class MarConfig(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int64), ("num_rels", ctypes.c_int32), ("dim", ctypes.c_int32),
                ("model", ctypes.c_int32), ("batch_size", ctypes.c_int32), ("num_chunks", ctypes.c_int32),
                ("negs_per_chunk", ctypes.c_int32), ("deg_negs_per_chunk", ctypes.c_int32),
                ("lr", ctypes.c_float), ("eps", ctypes.c_float), ("init_std", ctypes.c_float),
                ("seed", ctypes.c_uint64), ("precision", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class MarDebugOut(ctypes.Structure):
    _fields_ = [("num_uniq", ctypes.c_void_p), ("uniq_nodes", ctypes.c_void_p), ("uniq_rels", ctypes.c_void_p),
                ("pos", ctypes.c_void_p), ("lse_dst", ctypes.c_void_p), ("lse_src", ctypes.c_void_p),
                ("grad_rows", ctypes.c_void_p)]


EXPORTS = ("mar_workspace_bytes", "mar_init_tables", "mar_sample_negatives", "mar_train_batch", "mar_eval_scores",
           "mar_eval_filter", "mar_rank_metrics", "mar_rank_metrics_static", "mar_beta_buffer_sequence", "mar_beta_edge_bucket_order", "mar_buffer_simulate",
           "mar_swap_lower_bound", "mar_beta_swap_count",
           "mar_pipe_workspace_bytes", "mar_pipe_create", "mar_pipe_submit", "mar_pipe_drain", "mar_pipe_destroy",
           "mar_profile_enable", "mar_profile_read", "mar_destroy", "mar_last_error")


def library_path():
    return _LIB_PATH


def load_library():
    """Loads libmarius_hip.so (built in-tree by build.py); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError("%s not found: run `python -m paper_2101_08358_amd.build` (or __graft_entry__.build()) "
                                "first; there is no CPU fallback" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    lib.mar_workspace_bytes.argtypes = [ctypes.POINTER(MarConfig), ctypes.POINTER(ctypes.c_size_t)]
    lib.mar_init_tables.argtypes = [ctypes.POINTER(MarConfig), vp, vp, vp, vp, vp, ctypes.c_size_t, ctypes.c_int, vp,
                                    ctypes.POINTER(vp)]
    lib.mar_sample_negatives.argtypes = [vp, u64, vp, vp, i64, vp, vp, vp]
    lib.mar_train_batch.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, ctypes.POINTER(MarDebugOut), vp]
    lib.mar_eval_scores.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.mar_eval_filter.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.mar_rank_metrics.argtypes = [vp, vp, i64, ctypes.POINTER(i32), i32, vp, vp]
    lib.mar_rank_metrics_static.argtypes = [vp, i64, ctypes.POINTER(i32), i32, vp, vp]
    lib.mar_beta_buffer_sequence.argtypes = [i32, i32, vp, i64, ctypes.POINTER(i64)]
    lib.mar_beta_edge_bucket_order.argtypes = [i32, i32, i32, u64, vp]
    lib.mar_buffer_simulate.argtypes = [i32, i32, vp, i64, ctypes.POINTER(i64)]
    lib.mar_swap_lower_bound.argtypes = [i32, i32]
    lib.mar_beta_swap_count.argtypes = [i32, i32]
    lib.mar_pipe_workspace_bytes.argtypes = [ctypes.POINTER(MarConfig), i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.mar_pipe_create.argtypes = [ctypes.POINTER(MarConfig), vp, vp, vp, vp, vp, ctypes.c_size_t, i32, vp, ctypes.POINTER(vp)]
    lib.mar_pipe_submit.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.mar_pipe_drain.argtypes = [vp, vp]
    lib.mar_pipe_destroy.argtypes = [vp]
    lib.mar_profile_enable.argtypes = [vp, i32, ctypes.c_uint32]
    lib.mar_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.mar_destroy.argtypes = [vp]
    lib.mar_last_error.argtypes = [vp]
    lib.mar_last_error.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name in ("mar_swap_lower_bound", "mar_beta_swap_count"):
            getattr(lib, name).restype = ctypes.c_int64
        elif name != "mar_last_error":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise MarError(rc, load_library().mar_last_error(None).decode())


def _ptr(t):
    """Device (or NULL) pointer of a torch tensor / None / int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def mar_last_error():
    return load_library().mar_last_error(None).decode()


def mar_workspace_bytes(cfg):
    out = ctypes.c_size_t(0)
    _check(load_library().mar_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)))
    return out.value


def mar_init_tables(cfg, node_emb, node_state, rel_emb, rel_state, workspace, workspace_bytes, fill, stream=None):
    ctx = ctypes.c_void_p(None)
    _check(load_library().mar_init_tables(ctypes.byref(cfg), _ptr(node_emb), _ptr(node_state), _ptr(rel_emb),
                                          _ptr(rel_state), _ptr(workspace), workspace_bytes, int(fill),
                                          _stream(stream), ctypes.byref(ctx)))
    return ctx


def mar_sample_negatives(ctx, step, edge_src, edge_dst, num_edges, neg_src, neg_dst, stream=None):
    _check(load_library().mar_sample_negatives(ctx, int(step), _ptr(edge_src), _ptr(edge_dst), int(num_edges),
                                               _ptr(neg_src), _ptr(neg_dst), _stream(stream)))


def mar_train_batch(ctx, src, rel, dst, n_edges, neg_src, neg_dst, loss_sum_out=None, dbg=None, stream=None):
    _check(load_library().mar_train_batch(ctx, _ptr(src), _ptr(rel), _ptr(dst), int(n_edges), _ptr(neg_src),
                                          _ptr(neg_dst), _ptr(loss_sum_out),
                                          ctypes.byref(dbg) if dbg is not None else None, _stream(stream)))


def mar_eval_scores(ctx, src, rel, dst, n_edges, neg_src, neg_dst, pos_scores, rank_dst, rank_src, stream=None):
    _check(load_library().mar_eval_scores(ctx, _ptr(src), _ptr(rel), _ptr(dst), int(n_edges), _ptr(neg_src),
                                          _ptr(neg_dst), _ptr(pos_scores), _ptr(rank_dst), _ptr(rank_src),
                                          _stream(stream)))


def mar_eval_filter(ctx, src, rel, dst, n_edges, dst_off, dst_ids, src_off, src_ids, pos_scores, rank_dst, rank_src,
                    stream=None):
    _check(load_library().mar_eval_filter(ctx, _ptr(src), _ptr(rel), _ptr(dst), int(n_edges), _ptr(dst_off), _ptr(dst_ids),
                                          _ptr(src_off), _ptr(src_ids), _ptr(pos_scores), _ptr(rank_dst), _ptr(rank_src),
                                          _stream(stream)))


def mar_rank_metrics(ctx, ranks, n_ranks, ks, out, stream=None):
    arr = (ctypes.c_int32 * max(len(ks), 1))(*ks)
    _check(load_library().mar_rank_metrics(ctx, _ptr(ranks), int(n_ranks), arr, len(ks), _ptr(out), _stream(stream)))


def mar_rank_metrics_static(ranks, n_ranks, ks, out, stream=None):
    arr = (ctypes.c_int32 * max(len(ks), 1))(*ks)
    _check(load_library().mar_rank_metrics_static(_ptr(ranks), int(n_ranks), arr, len(ks), _ptr(out), _stream(stream)))


def mar_swap_lower_bound(p, c):
    return int(load_library().mar_swap_lower_bound(p, c))


def mar_beta_swap_count(p, c):
    return int(load_library().mar_beta_swap_count(p, c))


def mar_beta_buffer_sequence(p, c):
    """Returns the buffer sequence as a numpy int32 array [rows, c] (host memory)."""
    import numpy as np
    rows = ctypes.c_int64(0)
    _check(load_library().mar_beta_buffer_sequence(p, c, None, 0, ctypes.byref(rows)))
    out = np.empty((rows.value, c), dtype=np.int32)
    _check(load_library().mar_beta_buffer_sequence(p, c, out.ctypes.data, rows.value, ctypes.byref(rows)))
    return out


def mar_beta_edge_bucket_order(p, c, shuffle=False, seed=0):
    """Returns the edge-bucket order as a numpy int32 array [p*p, 2] (host memory)."""
    import numpy as np
    out = np.empty((p * p, 2), dtype=np.int32)
    _check(load_library().mar_beta_edge_bucket_order(p, c, 1 if shuffle else 0, int(seed), out.ctypes.data))
    return out


def mar_buffer_simulate(p, c, pairs):
    """Partition loads of replaying `pairs` ([n, 2] int32, host) through a buffer of c partitions."""
    import numpy as np
    arr = np.ascontiguousarray(pairs, dtype=np.int32)
    loads = ctypes.c_int64(0)
    _check(load_library().mar_buffer_simulate(p, c, arr.ctypes.data, arr.shape[0], ctypes.byref(loads)))
    return loads.value


def mar_pipe_workspace_bytes(cfg, depth):
    out = ctypes.c_size_t(0)
    _check(load_library().mar_pipe_workspace_bytes(ctypes.byref(cfg), int(depth), ctypes.byref(out)))
    return out.value


def mar_pipe_create(cfg, host_node_emb, host_node_state, rel_emb, rel_state, workspace, workspace_bytes, depth, stream=None):
    pipe = ctypes.c_void_p(None)
    _check(load_library().mar_pipe_create(ctypes.byref(cfg), _ptr(host_node_emb), _ptr(host_node_state), _ptr(rel_emb),
                                          _ptr(rel_state), _ptr(workspace), workspace_bytes, int(depth), _stream(stream),
                                          ctypes.byref(pipe)))
    return pipe


def mar_pipe_submit(pipe, src, rel, dst, n_edges, neg_src, neg_dst, loss_sum_out=None, ids_stream=None, stream=None):
    _check(load_library().mar_pipe_submit(pipe, _ptr(src), _ptr(rel), _ptr(dst), int(n_edges), _ptr(neg_src), _ptr(neg_dst),
                                          _ptr(loss_sum_out), _stream(ids_stream), _stream(stream)))


def mar_pipe_drain(pipe, stream=None):
    _check(load_library().mar_pipe_drain(pipe, _stream(stream)))


def mar_pipe_destroy(pipe):
    _check(load_library().mar_pipe_destroy(pipe))


def mar_profile_enable(ctx, max_steps, phase_mask=(1 << NUM_PHASES) - 1):
    _check(load_library().mar_profile_enable(ctx, int(max_steps), int(phase_mask)))


def mar_profile_read(ctx):
    ms = (ctypes.c_double * NUM_PHASES)()
    steps = ctypes.c_int32(0)
    _check(load_library().mar_profile_read(ctx, ms, ctypes.byref(steps)))
    return list(ms), steps.value


def mar_destroy(ctx):
    _check(load_library().mar_destroy(ctx))


class Trainer:
    """Owns the torch tensors (tables, workspace, id and output buffers) of one context.
    Convenience only: each method is one C-ABI call."""

    def __init__(self, num_nodes, num_rels, dim, model, batch_size, num_chunks, negs_per_chunk, deg_negs_per_chunk=0,
                 lr=0.1, eps=1e-10, init_std=0.001, seed=0, device="cuda:0", node_emb=None, rel_emb=None,
                 node_state=None, rel_state=None, precision=0):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.cfg = MarConfig(num_nodes, num_rels, dim, model, batch_size, num_chunks, negs_per_chunk,
                             deg_negs_per_chunk, lr, eps, init_std, seed, precision, 0)
        fill = node_emb is None
        f32 = dict(dtype=torch.float32, device=self.device)

        def table(rows, given):
            if given is None:
                return torch.empty((rows, dim), **f32)
            if torch.is_tensor(given) and given.device == self.device and given.dtype == torch.float32 \
                    and given.is_contiguous() and tuple(given.shape) == (rows, dim):
                return given                                    # adopt the caller's device tensor in place
            return torch.as_tensor(given, dtype=torch.float32).to(self.device).contiguous().clone()

        self.node_emb = table(num_nodes, node_emb)
        self.rel_emb = table(num_rels, rel_emb)
        self.node_state = table(num_nodes, node_state) if node_state is not None else (
            torch.empty((num_nodes, dim), **f32) if fill else torch.zeros((num_nodes, dim), **f32))
        self.rel_state = table(num_rels, rel_state) if rel_state is not None else (
            torch.empty((num_rels, dim), **f32) if fill else torch.zeros((num_rels, dim), **f32))
        self.workspace_bytes = mar_workspace_bytes(self.cfg)
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.device)
        with torch.cuda.device(self.device):
            self.ctx = mar_init_tables(self.cfg, self.node_emb, self.node_state, self.rel_emb, self.rel_state,
                                       self.workspace, self.workspace_bytes, 1 if fill else 0)
        cn = num_chunks * negs_per_chunk
        self.neg_src = torch.empty(cn, dtype=torch.int32, device=self.device)
        self.neg_dst = torch.empty(cn, dtype=torch.int32, device=self.device)
        self.loss = torch.zeros(1, **f32)

    def sample_negatives(self, step, edge_src=None, edge_dst=None):
        n = 0 if edge_src is None else edge_src.numel()
        mar_sample_negatives(self.ctx, step, edge_src, edge_dst, n, self.neg_src, self.neg_dst)

    def train_batch(self, src, rel, dst, dbg=None):
        mar_train_batch(self.ctx, src, rel, dst, src.numel(), self.neg_src, self.neg_dst, self.loss, dbg)
        return self.loss

    def make_debug(self, n_edges):
        """Allocates debug buffers; returns (struct, dict of tensors)."""
        torch = self.torch
        c = self.cfg
        cap = min(c.num_nodes + c.num_rels, 3 * c.batch_size + 2 * c.num_chunks * c.negs_per_chunk)
        i32 = dict(dtype=torch.int32, device=self.device)
        f32 = dict(dtype=torch.float32, device=self.device)
        t = dict(num_uniq=torch.zeros(2, **i32), uniq_nodes=torch.zeros(cap, **i32), uniq_rels=torch.zeros(cap, **i32),
                 pos=torch.zeros(max(n_edges, 1), **f32), lse_dst=torch.zeros(max(n_edges, 1), **f32),
                 lse_src=torch.zeros(max(n_edges, 1), **f32), grad_rows=torch.zeros(cap * c.dim, **f32))
        s = MarDebugOut(*[t[k].data_ptr() for k in ("num_uniq", "uniq_nodes", "uniq_rels", "pos", "lse_dst", "lse_src",
                                                    "grad_rows")])
        return s, t

    def eval_scores(self, src, rel, dst):
        torch = self.torch
        n = src.numel()
        pos = torch.empty(max(n, 1), dtype=torch.float32, device=self.device)
        rd = torch.empty(max(n, 1), dtype=torch.int32, device=self.device)
        rs = torch.empty(max(n, 1), dtype=torch.int32, device=self.device)
        mar_eval_scores(self.ctx, src, rel, dst, n, self.neg_src, self.neg_dst, pos, rd, rs)
        return pos[:n], rd[:n], rs[:n]

    def close(self):
        if self.ctx is not None:
            mar_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
