"""Thin ctypes binding of ``libhx.so`` with the names of ``include/hx.h``.

Argument marshalling only: every step of the search runs in the library's HIP
kernels.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhx.so")

HX_OK = 0
ERRORS = {-1: "HX_ERR_INVALID_ARG", -2: "HX_ERR_SHAPE", -3: "HX_ERR_NOT_DAG", -4: "HX_ERR_CAPACITY",
          -5: "HX_ERR_DEVICE", -6: "HX_ERR_INDEX", -7: "HX_ERR_OVERFLOW"}

EXPORTS = ("hx_ctx_create", "hx_ctx_destroy", "hx_last_error", "hx_stream_status", "hx_node_cost",
           "hx_critical_path", "hx_horizons", "hx_dag_reserve", "hx_dag_append", "hx_dag_set_cost", "hx_dag_view",
           "hx_score_placements", "hx_validate_round", "hx_select", "hx_urgency", "hx_commit", "hx_commit_static", "hx_round", "hx_rank", "hx_plan_greedy",
           "hx_decode_score", "hx_decode_plan_greedy")


class HxError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{ERRORS.get(code, code)}: {text}")
        self.code = code


class hx_model(C.Structure):
    _fields_ = [("kv_bytes_per_token", C.c_float), ("flops_per_token", C.c_float),
                ("attn_flops_per_token2", C.c_float), ("weight_bytes", C.c_float),
                ("nominal_batch", C.c_float)]


class hx_calls(C.Structure):
    _fields_ = [("n", C.c_int32), ("L_in", C.c_void_p), ("L_out", C.c_void_p), ("node", C.c_void_p),
                ("wf", C.c_void_p), ("elapsed", C.c_void_p)]


class hx_prefill_tab(C.Structure):
    _fields_ = [("n", C.c_int32), ("flops", C.c_void_p), ("hbm_bw", C.c_void_p),
                ("backlog_tok", C.c_void_p), ("type", C.c_void_p)]


class hx_decode_tab(C.Structure):
    _fields_ = [("n", C.c_int32), ("flops", C.c_void_p), ("hbm_bw", C.c_void_p), ("used_tok", C.c_void_p),
                ("cap_tok", C.c_void_p), ("batch", C.c_void_p), ("qd_tok", C.c_void_p), ("type", C.c_void_p)]


class hx_links(C.Structure):
    _fields_ = [("n_types", C.c_int32), ("bw", C.c_void_p), ("latency", C.c_void_p)]


class hx_intervals(C.Structure):
    _fields_ = [("stride", C.c_int32), ("count", C.c_void_p), ("start", C.c_void_p), ("end", C.c_void_p),
                ("tok", C.c_void_p)]


class hx_round_args(C.Structure):
    _fields_ = [("n_new", C.c_int32), ("n_new_edges", C.c_int32), ("parent_row_ptr", C.c_void_p), ("parent_col_idx", C.c_void_p),
                ("new_L_in", C.c_void_p), ("new_L_out", C.c_void_p), ("new_wf", C.c_void_p), ("new_cost", C.c_void_p),
                ("n_types", C.c_int32), ("type_flops", C.c_void_p), ("type_hbm_bw", C.c_void_p), ("n_wf", C.c_int32),
                ("n_nodes", C.c_int32), ("n_edges", C.c_int32), ("succ_row_ptr", C.c_void_p), ("succ_col_idx", C.c_void_p),
                ("wf_ptr", C.c_void_p), ("node_L_in", C.c_void_p), ("node_L_out", C.c_void_p),
                ("node_cost", C.c_void_p), ("rem", C.c_void_p), ("tail", C.c_void_p), ("level", C.c_void_p), ("horizon", C.c_void_p),
                ("calls", hx_calls), ("prefill", hx_prefill_tab), ("decode", hx_decode_tab), ("links", hx_links),
                ("best_p", C.c_void_p), ("best_d", C.c_void_p), ("best_cost", C.c_void_p), ("ratio", C.c_void_p),
                ("backlog_tok", C.c_void_p), ("used_tok", C.c_void_p), ("batch", C.c_void_p), ("qd_tok", C.c_void_p),
                ("drain_prefill", C.c_void_p), ("drain_decode_q", C.c_void_p), ("release_tok", C.c_void_p),
                ("tokens_per_seq", C.c_int32), ("max_batch", C.c_int32)]


_lib = None


def load() -> C.CDLL:
    """Loads the library (built in-tree by ``build.py``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2605_16637_amd.build` "
                              "(or __graft_entry__.build()) first")
        # PyTorch ships its own copy of the HIP runtime; import it first so the
        # library binds to that copy and the process holds exactly one runtime
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name).restype = C.c_int
        lib.hx_last_error.restype = C.c_char_p
        _lib = lib
    return _lib


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("the placement search needs a GPU: no HIP device is visible")
    return torch


class RawArray:
    """A device array known only by address (e.g. one returned by hx_dag_view)."""

    def __init__(self, addr: int, numel: int, dtype):
        self.addr, self._n, self.dtype = int(addr), int(numel), dtype

    def numel(self):
        return self._n


def _ptr(t, dtype=None, n=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL), after checks."""
    if t is None:
        return None
    if isinstance(t, RawArray):
        if dtype is not None and t.dtype != dtype:
            raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
        if n is not None and t.numel() < n:
            raise ValueError(f"array has {t.numel()} elements, {n} needed")
        return C.c_void_p(t.addr)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous tensor in device memory")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    if n is not None and t.numel() < n:
        raise ValueError(f"tensor has {t.numel()} elements, {n} needed")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def make_model(m: dict) -> hx_model:
    return hx_model(m["kv_bytes_per_token"], m["flops_per_token"], m["attn_flops_per_token2"],
                    m["weight_bytes"], m["nominal_batch"])


def make_calls(c: dict) -> hx_calls:
    torch = _torch()
    n = int(c["n"])
    return hx_calls(n, _ptr(c["L_in"], torch.int32, n), _ptr(c["L_out"], torch.int32, n),
                    _ptr(c.get("node"), torch.int32, n), _ptr(c.get("wf"), torch.int32, n),
                    _ptr(c.get("elapsed"), torch.float32, n))


def make_prefill(p: dict) -> hx_prefill_tab:
    torch = _torch()
    n = int(p["n"])
    return hx_prefill_tab(n, _ptr(p["flops"], torch.float32, n), _ptr(p["hbm_bw"], torch.float32, n),
                          _ptr(p["backlog_tok"], torch.int32, n), _ptr(p["type"], torch.int32, n))


def make_decode(d: dict) -> hx_decode_tab:
    torch = _torch()
    n = int(d["n"])
    i32 = torch.int32
    return hx_decode_tab(n, _ptr(d["flops"], torch.float32, n), _ptr(d["hbm_bw"], torch.float32, n),
                         _ptr(d["used_tok"], i32, n), _ptr(d["cap_tok"], i32, n), _ptr(d["batch"], i32, n),
                         _ptr(d["qd_tok"], i32, n), _ptr(d["type"], i32, n))


def make_links(l: dict) -> hx_links:
    torch = _torch()
    T = int(l["n_types"])
    return hx_links(T, _ptr(l["bw"], torch.float32, T * T), _ptr(l.get("latency"), torch.float32, T * T))


def make_intervals(iv: dict, D: int) -> hx_intervals:
    torch = _torch()
    k = int(iv["stride"])
    return hx_intervals(k, _ptr(iv["count"], torch.int32, D), _ptr(iv["start"], torch.float32, D * k),
                        _ptr(iv["end"], torch.float32, D * k), _ptr(iv["tok"], torch.int32, D * k))


class Context:
    """Owns one ``hx_ctx``.  Methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0):
        torch = _torch()
        # the HIP runtime in this process is PyTorch's copy; let PyTorch bring the
        # device up before the library makes its first HIP call
        torch.cuda.init()
        torch.empty(1, device=f"cuda:{int(device)}")
        self.lib = load()
        self._ctx = C.c_void_p()
        rc = self.lib.hx_ctx_create(C.byref(self._ctx), int(device))
        if rc != HX_OK:
            raise HxError(rc, self.lib.hx_last_error(None).decode())
        self.device = device
        self._recording = None

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self.lib.hx_ctx_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != HX_OK:
            raise HxError(rc, self.lib.hx_last_error(self._ctx).decode())

    def _invoke(self, fn, *args):
        """Calls an entry point with marshalled arguments -- or, inside prepare(), only notes the call."""
        if self._recording is not None:
            self._recording.append((fn, args))
        else:
            self._check(fn(*args))

    def prepare(self, fn):
        """Runs ``fn`` (any sequence of this context's calls) without calling the library and returns a
        callable that makes exactly those library calls with the arguments marshalled now: for loops where
        the same calls recur on the same buffers (a scheduling round replayed every few tens of microseconds)
        and the marshalling would cost more than the launches.  The tensors passed must stay alive and in
        place; the stream is the one current at prepare time.  Calls that return values (hx_dag_view,
        hx_validate_round) are made as usual."""
        self._recording = []
        try:
            fn()
            calls = self._recording
        finally:
            self._recording = None
        ctx, last_error = self._ctx, self.lib.hx_last_error

        def replay():
            for f, a in calls:
                rc = f(*a)
                if rc != HX_OK:
                    raise HxError(rc, last_error(ctx).decode())
        replay.n_calls = len(calls)
        return replay

    def hx_stream_status(self, stream=None):
        self._invoke(self.lib.hx_stream_status, self._ctx, _stream(stream))

    def hx_node_cost(self, model, L_in, L_out, type_flops, type_hbm_bw, links, cost, stream=None):
        torch = _torch()
        n, T = int(L_in.numel()), int(type_flops.numel())
        m, lk = make_model(model), make_links(links)
        self._invoke(self.lib.hx_node_cost, self._ctx, C.byref(m), n, _ptr(L_in, torch.int32), _ptr(L_out, torch.int32, n),
                                          T, _ptr(type_flops, torch.float32), _ptr(type_hbm_bw, torch.float32, T),
                                          C.byref(lk), _ptr(cost, torch.float32, n), _stream(stream))

    def hx_critical_path(self, succ_row_ptr, succ_col_idx, node_cost, wf_ptr, rem, tail, level, horizon,
                         max_sweeps=0, stream=None):
        torch = _torch()
        n, n_wf, n_edges = int(succ_row_ptr.numel()) - 1, int(wf_ptr.numel()) - 1, int(succ_col_idx.numel())
        self._invoke(self.lib.hx_critical_path, 
            self._ctx, n, n_edges, _ptr(succ_row_ptr, torch.int32), _ptr(succ_col_idx, torch.int32),
            _ptr(node_cost, torch.float32, n), n_wf, _ptr(wf_ptr, torch.int32), int(max_sweeps),
            _ptr(rem, torch.float32, n), _ptr(tail, torch.float32, n), _ptr(level, torch.int32, n),
            _ptr(horizon, torch.float32, n_wf), _stream(stream))

    def hx_horizons(self, model, succ_row_ptr, succ_col_idx, L_in, L_out, type_flops, type_hbm_bw, links, wf_ptr,
                    node_cost, rem, tail, level, horizon, stream=None):
        torch = _torch()
        n, n_wf, n_edges = int(succ_row_ptr.numel()) - 1, int(wf_ptr.numel()) - 1, int(succ_col_idx.numel())
        T = int(type_flops.numel())
        m, lk = make_model(model), make_links(links)
        self._invoke(self.lib.hx_horizons, 
            self._ctx, C.byref(m), n, n_edges, _ptr(succ_row_ptr, torch.int32), _ptr(succ_col_idx, torch.int32),
            _ptr(L_in, torch.int32, n), _ptr(L_out, torch.int32, n), T, _ptr(type_flops, torch.float32),
            _ptr(type_hbm_bw, torch.float32, T), C.byref(lk), n_wf, _ptr(wf_ptr, torch.int32),
            _ptr(node_cost, torch.float32, n), _ptr(rem, torch.float32, n), _ptr(tail, torch.float32, n),
            _ptr(level, torch.int32, n), _ptr(horizon, torch.float32, n_wf), _stream(stream))

    def hx_dag_reserve(self, max_nodes, max_edges, max_wf, max_depth, stream=None):
        self._invoke(self.lib.hx_dag_reserve, self._ctx, int(max_nodes), int(max_edges), int(max_wf),
                                            int(max_depth), _stream(stream))

    def hx_dag_append(self, parent_row_ptr, parent_col_idx, new_cost, new_wf, stream=None):
        torch = _torch()
        n_new, n_e = int(new_cost.numel()), int(parent_col_idx.numel())
        self._invoke(self.lib.hx_dag_append, self._ctx, n_new, n_e, _ptr(parent_row_ptr, torch.int32, n_new + 1),
                                           _ptr(parent_col_idx, torch.int32), _ptr(new_cost, torch.float32),
                                           _ptr(new_wf, torch.int32, n_new), _stream(stream))

    def hx_dag_set_cost(self, node_ids, cost, stream=None):
        torch = _torch()
        n = int(node_ids.numel())
        self._invoke(self.lib.hx_dag_set_cost, self._ctx, n, _ptr(node_ids, torch.int32), _ptr(cost, torch.float32, n), _stream(stream))

    def hx_dag_view(self, n_wf: int):
        """(rem, tail, level, horizon) of the context's graph as borrowed RawArray
        views (rem/tail/level over the nodes appended so far, horizon over the
        first n_wf workflows) and the node count."""
        torch = _torch()
        rem, tail, level, hor = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
        n = C.c_int32()
        self._check(self.lib.hx_dag_view(self._ctx, C.byref(rem), C.byref(tail), C.byref(level),
                                         C.byref(hor), C.byref(n)))
        return (RawArray(rem.value, n.value, torch.float32), RawArray(tail.value, n.value, torch.float32),
                RawArray(level.value, n.value, torch.int32), RawArray(hor.value, n_wf, torch.float32), n.value)

    def hx_score_placements(self, model, calls, prefill, decode, links, tail=None, horizon=None,
                            cost=None, feas=None, best_p=None, best_d=None, best_cost=None, ratio=None,
                            stream=None):
        torch = _torch()
        m, cs, pt, dt, lk = make_model(model), make_calls(calls), make_prefill(prefill), make_decode(decode), make_links(links)
        Cn, P, D = cs.n, pt.n, dt.n
        n_nodes = 0 if tail is None else int(tail.numel())
        n_wf = 0 if horizon is None else int(horizon.numel())
        self._invoke(self.lib.hx_score_placements, 
            self._ctx, C.byref(m), C.byref(cs), C.byref(pt), C.byref(dt), C.byref(lk),
            _ptr(tail, torch.float32), _ptr(horizon, torch.float32), n_nodes, n_wf,
            _ptr(cost, torch.float32, Cn * P * D), _ptr(feas, torch.uint8, Cn * D),
            _ptr(best_p, torch.int32, Cn), _ptr(best_d, torch.int32, Cn), _ptr(best_cost, torch.float32, Cn),
            _ptr(ratio, torch.float32, Cn), _stream(stream))

    VALIDATE_FIELDS = ("L_in", "L_out", "node", "wf", "elapsed", "prefill_rate", "prefill_backlog", "prefill_type",
                       "decode_rate", "decode_state", "decode_type", "link")

    def hx_validate_round(self, calls, prefill, decode, links, n_nodes=0, n_wf=0, stream=None):
        """Counts of out-of-range input elements per category (a dict); raises HxError if any is non-zero
        unless the caller reads the counts from the exception's ``report``."""
        cs, pt, dt, lk = make_calls(calls), make_prefill(prefill), make_decode(decode), make_links(links)
        report = (C.c_int32 * len(self.VALIDATE_FIELDS))()
        rc = self.lib.hx_validate_round(self._ctx, C.byref(cs), C.byref(pt), C.byref(dt), C.byref(lk),
                                        int(n_nodes), int(n_wf), report, _stream(stream))
        counts = dict(zip(self.VALIDATE_FIELDS, list(report)))
        if rc != HX_OK:
            err = HxError(rc, self.lib.hx_last_error(self._ctx).decode())
            err.report = counts
            raise err
        return counts

    def hx_select(self, C_, P, D, cost, best_p, best_d, best_cost, calls=None, tail=None, horizon=None,
                  ratio=None, stream=None):
        torch = _torch()
        cs = make_calls(calls) if calls is not None else None
        n_nodes = 0 if tail is None else int(tail.numel())
        n_wf = 0 if horizon is None else int(horizon.numel())
        self._invoke(self.lib.hx_select, 
            self._ctx, int(C_), int(P), int(D), _ptr(cost, torch.float32, C_ * P * D),
            C.byref(cs) if cs is not None else None, _ptr(tail, torch.float32), _ptr(horizon, torch.float32),
            n_nodes, n_wf, _ptr(best_p, torch.int32, C_), _ptr(best_d, torch.int32, C_),
            _ptr(best_cost, torch.float32, C_), _ptr(ratio, torch.float32, C_), _stream(stream))

    def hx_urgency(self, calls, best_cost, tail, horizon, ratio, stream=None):
        torch = _torch()
        cs = make_calls(calls)
        self._invoke(self.lib.hx_urgency, self._ctx, C.byref(cs), _ptr(best_cost, torch.float32, cs.n),
                                        _ptr(tail, torch.float32), _ptr(horizon, torch.float32),
                                        int(tail.numel()), int(horizon.numel()), _ptr(ratio, torch.float32, cs.n), _stream(stream))

    def hx_commit(self, calls, best_p, best_d, backlog_tok, used_tok, batch, qd_tok,
                  drain_prefill=None, drain_decode_q=None, release_tok=None,
                  tokens_per_seq=2048, max_batch=256, stream=None):
        torch = _torch()
        cs = make_calls(calls)
        P, D = int(backlog_tok.numel()), int(used_tok.numel())
        i32 = torch.int32
        self._invoke(self.lib.hx_commit, 
            self._ctx, C.byref(cs), _ptr(best_p, i32, cs.n), _ptr(best_d, i32, cs.n),
            P, _ptr(backlog_tok, i32), D, _ptr(used_tok, i32), _ptr(batch, i32, D), _ptr(qd_tok, i32, D),
            _ptr(drain_prefill, i32, P), _ptr(drain_decode_q, i32, D), _ptr(release_tok, i32, D),
            int(tokens_per_seq), int(max_batch), _stream(stream))


    def hx_round(self, model, calls, prefill, decode, links, best_p, best_d, best_cost, ratio=None, n_wf=0,
                 parent_row_ptr=None, parent_col_idx=None, new_L_in=None, new_L_out=None, new_wf=None, new_cost=None,
                 type_flops=None, type_hbm_bw=None, drain_prefill=None, drain_decode_q=None, release_tok=None,
                 tokens_per_seq=2048, max_batch=256, graph=None, stream=None):
        """One scheduling invocation in one library call: reveal (node cost + append, or -- ``graph``: a dict with
        succ_row_ptr, succ_col_idx, wf_ptr, L_in, L_out and the outputs node_cost, rem, tail, level, horizon --
        the whole graph's horizons), fused search with the ratio, commit into the pool's own counters."""
        torch = _torch()
        i32, f32 = torch.int32, torch.float32
        m = make_model(model)
        r = hx_round_args()
        n_new = 0 if new_L_in is None else int(new_L_in.numel())
        r.n_new, r.n_new_edges = n_new, 0 if parent_col_idx is None else int(parent_col_idx.numel())
        r.parent_row_ptr, r.parent_col_idx = _ptr(parent_row_ptr, i32, n_new + 1 if n_new else None), _ptr(parent_col_idx, i32)
        r.new_L_in, r.new_L_out, r.new_wf = _ptr(new_L_in, i32), _ptr(new_L_out, i32, n_new), _ptr(new_wf, i32, n_new)
        r.new_cost = _ptr(new_cost, f32, n_new)
        r.n_types = 0 if type_flops is None else int(type_flops.numel())
        r.type_flops, r.type_hbm_bw = _ptr(type_flops, f32), _ptr(type_hbm_bw, f32, r.n_types)
        r.n_wf = int(n_wf)
        if graph is not None:
            g = graph
            n, nw = int(g["succ_row_ptr"].numel()) - 1, int(g["wf_ptr"].numel()) - 1
            r.n_nodes, r.n_edges, r.n_wf = n, int(g["succ_col_idx"].numel()), nw
            r.succ_row_ptr, r.succ_col_idx, r.wf_ptr = _ptr(g["succ_row_ptr"], i32), _ptr(g["succ_col_idx"], i32), _ptr(g["wf_ptr"], i32)
            r.node_L_in, r.node_L_out = _ptr(g["L_in"], i32, n), _ptr(g["L_out"], i32, n)
            r.node_cost, r.rem, r.tail = _ptr(g["node_cost"], f32, n), _ptr(g["rem"], f32, n), _ptr(g["tail"], f32, n)
            r.level, r.horizon = _ptr(g["level"], i32, n), _ptr(g["horizon"], f32, nw)
        r.calls, r.prefill, r.decode, r.links = make_calls(calls), make_prefill(prefill), make_decode(decode), make_links(links)
        n = r.calls.n
        r.best_p, r.best_d, r.best_cost, r.ratio = _ptr(best_p, i32, n), _ptr(best_d, i32, n), _ptr(best_cost, f32, n), _ptr(ratio, f32, n)
        r.backlog_tok = _ptr(prefill["backlog_tok"], i32, r.prefill.n)
        r.used_tok, r.batch, r.qd_tok = (_ptr(decode[k], i32, r.decode.n) for k in ("used_tok", "batch", "qd_tok"))
        r.drain_prefill, r.drain_decode_q, r.release_tok = _ptr(drain_prefill, i32, r.prefill.n), _ptr(drain_decode_q, i32, r.decode.n), _ptr(release_tok, i32, r.decode.n)
        r.tokens_per_seq, r.max_batch = int(tokens_per_seq), int(max_batch)
        self._invoke(self.lib.hx_round, self._ctx, C.byref(m), C.byref(r), _stream(stream))

    def hx_rank(self, ratio, rank, stream=None):
        torch = _torch()
        n = int(ratio.numel())
        self._invoke(self.lib.hx_rank, self._ctx, n, _ptr(ratio, torch.float32), _ptr(rank, torch.int32, n), _stream(stream))

    def hx_plan_greedy(self, model, calls, prefill, decode, links, tail, horizon,
                       best_p, best_d, best_cost, ratio, rank,
                       backlog_tok_out=None, used_tok_out=None, batch_out=None, qd_tok_out=None,
                       tokens_per_seq=2048, max_batch=256, stream=None):
        torch = _torch()
        m, cs, pt, dt, lk = make_model(model), make_calls(calls), make_prefill(prefill), make_decode(decode), make_links(links)
        i32 = torch.int32
        self._invoke(self.lib.hx_plan_greedy, 
            self._ctx, C.byref(m), C.byref(cs), C.byref(pt), C.byref(dt), C.byref(lk),
            _ptr(tail, torch.float32), _ptr(horizon, torch.float32), int(tail.numel()), int(horizon.numel()),
            int(tokens_per_seq), int(max_batch),
            _ptr(best_p, i32, cs.n), _ptr(best_d, i32, cs.n), _ptr(best_cost, torch.float32, cs.n),
            _ptr(ratio, torch.float32, cs.n), _ptr(rank, i32, cs.n),
            _ptr(backlog_tok_out, i32, pt.n), _ptr(used_tok_out, i32, dt.n), _ptr(batch_out, i32, dt.n),
            _ptr(qd_tok_out, i32, dt.n), _stream(stream))


    def hx_decode_score(self, model, queue, lock, decode, intervals, best_d, best_start, best_cost,
                        tail=None, horizon=None, ratio=None, start=None, cost=None, stream=None):
        torch = _torch()
        m, cs, dt = make_model(model), make_calls(queue), make_decode(decode)
        iv = make_intervals(intervals, dt.n)
        n_nodes = 0 if tail is None else int(tail.numel())
        n_wf = 0 if horizon is None else int(horizon.numel())
        f32, i32 = torch.float32, torch.int32
        self._invoke(self.lib.hx_decode_score, 
            self._ctx, C.byref(m), C.byref(cs), _ptr(lock, i32, cs.n), C.byref(dt), C.byref(iv),
            _ptr(tail, f32), _ptr(horizon, f32), n_nodes, n_wf,
            _ptr(start, f32, cs.n * dt.n), _ptr(cost, f32, cs.n * dt.n),
            _ptr(best_d, i32, cs.n), _ptr(best_start, f32, cs.n), _ptr(best_cost, f32, cs.n), _ptr(ratio, f32, cs.n),
            _stream(stream))

    def hx_decode_plan_greedy(self, model, queue, lock, decode, intervals, tail, horizon,
                              best_d, best_start, best_cost, ratio, rank, stream=None):
        torch = _torch()
        m, cs, dt = make_model(model), make_calls(queue), make_decode(decode)
        iv = make_intervals(intervals, dt.n)
        f32, i32 = torch.float32, torch.int32
        self._invoke(self.lib.hx_decode_plan_greedy, 
            self._ctx, C.byref(m), C.byref(cs), _ptr(lock, i32, cs.n), C.byref(dt), C.byref(iv),
            _ptr(tail, f32), _ptr(horizon, f32), int(tail.numel()), int(horizon.numel()),
            _ptr(best_d, i32, cs.n), _ptr(best_start, f32, cs.n), _ptr(best_cost, f32, cs.n), _ptr(ratio, f32, cs.n),
            _ptr(rank, i32, cs.n), _stream(stream))


def hx_commit_static(calls, best_p, best_d, backlog_tok, used_tok, batch, qd_tok,
                     drain_prefill=None, drain_decode_q=None, release_tok=None,
                     tokens_per_seq=2048, max_batch=256, status=None, stream=None):
    """The commit that needs no context and allocates nothing (static scratch inside the library)."""
    torch = _torch()
    lib = load()
    cs = make_calls(calls)
    P, D = int(backlog_tok.numel()), int(used_tok.numel())
    i32 = torch.int32
    rc = lib.hx_commit_static(
        C.byref(cs), _ptr(best_p, i32, cs.n), _ptr(best_d, i32, cs.n),
        P, _ptr(backlog_tok, i32), D, _ptr(used_tok, i32), _ptr(batch, i32, D), _ptr(qd_tok, i32, D),
        _ptr(drain_prefill, i32, P), _ptr(drain_decode_q, i32, D), _ptr(release_tok, i32, D),
        int(tokens_per_seq), int(max_batch), _ptr(status, i32, 1), _stream(stream))
    if rc != HX_OK:
        raise HxError(rc, lib.hx_last_error(None).decode())


def to_device(d: dict, device="cuda:0") -> dict:
    """numpy tables of ``synth`` -> torch tensors in device memory (scalars and None pass through)."""
    import numpy as np
    torch = _torch()
    out = {}
    for k, v in d.items():
        if isinstance(v, np.ndarray):
            out[k] = torch.from_numpy(np.ascontiguousarray(v)).to(device)
        else:
            out[k] = v
    return out
