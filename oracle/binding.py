"""ctypes binding of oracle/mt_oracle.c.  Marshalling only; no arithmetic here."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import build

_lib = None


class _Cfg(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("max_pos", C.c_int32), ("type_vocab", C.c_int32), ("n_trunk_layers", C.c_int32),
                ("n_tasks", C.c_int32), ("gelu_tanh", C.c_int32), ("ln_eps", C.c_float)]


class _Task(C.Structure):
    _fields_ = [("fork_layer", C.c_int32), ("n_layers", C.c_int32), ("n_classes", C.c_int32), ("token_level", C.c_int32)]


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float)) if a is not None else None


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def lib():
    global _lib
    if _lib is None:
        # ORC_LIB: a library built elsewhere from a (deliberately altered) copy of the source; the mutation audit of the
        # pins uses it, nothing else does
        L = C.CDLL(os.environ.get("ORC_LIB") or build())
        L.orc_layer_param_count.restype = C.c_int64
        L.orc_layer_param_count.argtypes = [C.c_int64, C.c_int64]
        L.orc_trunk_param_count.restype = C.c_int64
        L.orc_task_param_count.restype = C.c_int64
        L.orc_gelu.restype = C.c_float
        L.orc_gelu.argtypes = [C.c_float, C.c_int]
        L.orc_overhead.restype = C.c_int
        L.orc_mt_forward.restype = C.c_int
        L.orc_st_forward.restype = C.c_int
        L.orc_mt_forward_typed.restype = C.c_int
        L.orc_mt_forward_tokens.restype = C.c_int
        L.orc_st_forward_typed.restype = C.c_int
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def set_num_threads(n: int) -> None:
    """Limit the OpenMP threads the oracle uses from now on (timing baselines only; results do not depend on it)."""
    lib().orc_set_num_threads(int(n))


def num_threads() -> int:
    """Threads the oracle's OpenMP loops will use."""
    return int(lib().orc_num_threads())


def layer_param_count(h: int, f: int) -> int:
    return int(lib().orc_layer_param_count(h, f))


def overhead(tasks) -> int:
    """tasks: iterable of (fork_layer x, n_layers y[, n_classes])."""
    arr = (_Task * len(tasks))(*[_Task(int(t[0]), int(t[1]), int(t[2]) if len(t) > 2 else 1, 0) for t in tasks])
    return int(lib().orc_overhead(arr, C.c_int(len(tasks))))


def linear(x, w, b=None):
    x, w = _f32(x), _f32(w)
    m, k = x.shape
    n = w.shape[0]
    assert w.shape[1] == k
    bb = _f32(b) if b is not None else None
    y = np.empty((m, n), dtype=np.float32)
    lib().orc_linear(_fp(x), C.c_int64(m), C.c_int64(k), _fp(w), _fp(bb), C.c_int64(n), _fp(y))
    return y


def layernorm(x, gamma, beta, eps=1e-12, residual=None):
    x = _f32(x)
    m, h = x.shape
    r = _f32(residual) if residual is not None else None
    g, bt = _f32(gamma), _f32(beta)
    y = np.empty_like(x)
    lib().orc_layernorm(_fp(x), _fp(r), C.c_int64(m), C.c_int64(h), _fp(g), _fp(bt), C.c_float(eps), _fp(y))
    return y


def gelu(x, tanh_form=False):
    x = _f32(x)
    y = np.empty_like(x)
    lib().orc_gelu_array(_fp(x), C.c_int64(x.size), C.c_int(int(tanh_form)), _fp(y))
    return y


def softmax_row(s):
    s = _f32(s).ravel()
    p = np.empty_like(s)
    lib().orc_softmax_row(_fp(s), C.c_int64(s.size), _fp(p))
    return p


def attention(q, k, v, mask, heads, want_probs=False):
    q, k, v, mask = _f32(q), _f32(k), _f32(v), _i32(mask)
    b, s, h = q.shape
    ctx = np.empty_like(q)
    probs = np.empty((b, heads, s, s), dtype=np.float32) if want_probs else None
    lib().orc_attention(_fp(q), _fp(k), _fp(v), _ip(mask), C.c_int64(b), C.c_int64(s), C.c_int64(h),
                        C.c_int64(heads), _fp(ctx), _fp(probs))
    return (ctx, probs) if want_probs else ctx


def _cfg_of(spec) -> _Cfg:
    return _Cfg(spec.vocab, spec.hidden, spec.heads, spec.ffn, spec.max_pos, spec.type_vocab,
                spec.n_trunk_layers, len(spec.tasks), 1 if spec.gelu == "tanh" else 0, spec.ln_eps)


def encoder_layer(spec, layer_params, x, mask):
    """One encoder layer; layer_params is the flat canonical parameter vector of that layer."""
    x, mask, lp = _f32(x), _i32(mask), _f32(layer_params)
    b, s, h = x.shape
    assert lp.size == layer_param_count(spec.hidden, spec.ffn)
    cfg = _cfg_of(spec)
    out = np.empty_like(x)
    lib().orc_encoder_layer(C.byref(cfg), _fp(lp), _fp(x), _ip(mask), C.c_int64(b), C.c_int64(s), _fp(out))
    return out


class Oracle:
    """The merged model (mt_forward) and each student on its own (st_forward) for one spec + weights."""

    def __init__(self, spec, trunk_params, task_params):
        self.spec = spec
        self.cfg = _cfg_of(spec)
        self.tasks = (_Task * len(spec.tasks))(*[_Task(t.fork_layer, t.n_layers, t.n_classes, int(getattr(t, "token_level", False)))
                                               for t in spec.tasks])
        self.trunk = _f32(trunk_params)
        self.task_params = [_f32(p) for p in task_params]
        L = lib()
        assert self.trunk.size == L.orc_trunk_param_count(C.byref(self.cfg)), "trunk parameter count"
        for t, p in enumerate(self.task_params):
            assert p.size == L.orc_task_param_count(C.byref(self.cfg), C.byref(self.tasks[t])), f"task {t} parameter count"

    def mt_forward(self, ids, mask, want_hidden=False, type_ids=None, want_tokens=False):
        """type_ids: optional [B,S] segment ids in [0, type_vocab); None = segment 0 everywhere.
        want_tokens: also return the token-level tasks' logits [B,S,n_token_logits] (after the per-sequence ones)."""
        ids, mask = _i32(ids), _i32(mask)
        tt = _i32(type_ids) if type_ids is not None else None
        b, s = ids.shape
        sp = self.spec
        logits = np.empty((b, sp.n_logits), dtype=np.float32)
        n_tok = sum(t.n_classes for t in sp.tasks if getattr(t, "token_level", False))
        tok = np.empty((b, s, n_tok), dtype=np.float32)
        hidden = np.empty((sp.n_trunk_layers + 1, b, s, sp.hidden), dtype=np.float32) if want_hidden else None
        ptrs = (C.POINTER(C.c_float) * len(self.task_params))(*[_fp(p) for p in self.task_params])
        rc = lib().orc_mt_forward_tokens(C.byref(self.cfg), self.tasks, _fp(self.trunk), ptrs, _ip(ids),
                                         _ip(tt) if tt is not None else None, _ip(mask),
                                         C.c_int64(b), C.c_int64(s), _fp(logits) if logits.size else None,
                                         _fp(tok) if n_tok else None, _fp(hidden))
        if rc != 0:
            raise ValueError("invalid task table")
        res = (logits,) + ((tok,) if want_tokens else ()) + ((hidden,) if want_hidden else ())
        return res if len(res) > 1 else logits

    def st_forward(self, t, ids, mask, type_ids=None):
        ids, mask = _i32(ids), _i32(mask)
        tt = _i32(type_ids) if type_ids is not None else None
        b, s = ids.shape
        task = self.spec.tasks[t]
        shape = (b, s, task.n_classes) if getattr(task, "token_level", False) else (b, task.n_classes)
        logits = np.empty(shape, dtype=np.float32)
        rc = lib().orc_st_forward_typed(C.byref(self.cfg), C.byref(self.tasks[t]), _fp(self.trunk), _fp(self.task_params[t]),
                                        _ip(ids), _ip(tt) if tt is not None else None, _ip(mask), C.c_int64(b), C.c_int64(s),
                                        _fp(logits))
        if rc != 0:
            raise ValueError("invalid task")
        return logits
