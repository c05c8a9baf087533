"""ctypes binding of libmt_hip.so with the C ABI's names (include/mt.h).  Marshalling only.

PyTorch appears here solely as the owner of device memory and streams: arenas are torch tensors
whose data_ptr() is handed to the library, and the stream handle is torch's current HIP stream.
There is no fallback: if the shared library is missing or cannot be loaded, importing a symbol
raises.
"""
from __future__ import annotations

import ctypes as C
import os
import struct

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmt_hip.so")

MT_OK, MT_ERR_NULL, MT_ERR_CONFIG, MT_ERR_SHAPE, MT_ERR_STATE, MT_ERR_BLOB, MT_ERR_HIP = 0, -1, -2, -3, -4, -5, -6
MT_BF16, MT_FP32_CHECK, MT_FP8_FFN, MT_FP8_LAYER = 0, 1, 2, 3
MT_GELU_ERF, MT_GELU_TANH = 0, 1
MT_ABI_VERSION = 2
MT_HEAD_SEQUENCE, MT_HEAD_TOKEN = 0, 1
KERNEL_CLASSES = ["embed", "gemm_qkv", "attn", "gemm_out", "ln", "gemm_ffn1", "gemm_ffn2", "pool", "gemm_first"]

EXPORTS = ["mt_create", "mt_destroy", "mt_weight_bytes", "mt_workspace_bytes", "mt_bind", "mt_load_weights",
           "mt_forward", "mt_logit_offset", "mt_n_logits", "mt_layer_count", "mt_last_error", "mt_error_name",
           "mt_read_hidden", "mt_profile_enable", "mt_profile_read", "mt_op_linear", "mt_op_attention",
           "mt_op_layernorm", "mt_op_linear_batched", "mt_debug_set_gemm_tile", "mt_share_weights", "mt_debug_mfma_peak", "mt_forward_typed", "mt_op_linear_sub", "mt_op_first_token_pool", "mt_schedule_steps", "mt_forward_routed",
           "mt_forward_tokens", "mt_token_logit_offset", "mt_n_token_logits", "mt_forward_static", "mt_forward_multi", "mt_forward_requests", "mt_forward_routed_tokens", "mt_op_linear_fp8", "mt_debug_e4m3_quantize", "mt_check_mask"]
MT_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


class mt_task_desc(C.Structure):
    _fields_ = [("fork_layer", C.c_int32), ("n_layers", C.c_int32), ("n_classes", C.c_int32), ("head", C.c_int32)]


class mt_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("version", C.c_uint32),
                ("vocab", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("max_pos", C.c_int32), ("type_vocab", C.c_int32), ("n_trunk_layers", C.c_int32),
                ("n_tasks", C.c_int32), ("tasks", C.POINTER(mt_task_desc)),
                ("precision", C.c_int32), ("gelu", C.c_int32), ("ln_eps", C.c_float),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32)]


_lib = None


def lib():
    """Load libmt_hip.so (built in-tree by build.py); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.mt_create.argtypes = [C.POINTER(mt_config), C.POINTER(vp)]
        L.mt_destroy.argtypes = [vp]
        L.mt_destroy.restype = None
        L.mt_weight_bytes.argtypes = [vp]
        L.mt_weight_bytes.restype = sz
        L.mt_workspace_bytes.argtypes = [vp]
        L.mt_workspace_bytes.restype = sz
        L.mt_bind.argtypes = [vp, vp, sz, vp, sz]
        L.mt_load_weights.argtypes = [vp, i32, vp, sz, vp]
        L.mt_forward.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
        L.mt_forward_static.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
        L.mt_forward_multi.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp, vp]
        L.mt_forward_requests.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, vp]
        L.mt_forward_typed.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.mt_forward_routed.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.mt_forward_tokens.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        L.mt_forward_routed_tokens.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        L.mt_check_mask.argtypes = [vp, vp, i32, i32, C.POINTER(C.c_int32), vp]
        L.mt_op_linear_fp8.argtypes = [vp, i64, vp, C.c_float, vp, vp, vp, i64, i32, i32, i32, i32, i32, C.c_float, vp]
        L.mt_debug_e4m3_quantize.argtypes = [vp, sz, vp]
        L.mt_debug_e4m3_quantize.restype = C.c_float
        L.mt_logit_offset.argtypes = [vp, i32]
        L.mt_token_logit_offset.argtypes = [vp, i32]
        L.mt_n_token_logits.argtypes = [vp]
        L.mt_n_logits.argtypes = [vp]
        L.mt_layer_count.argtypes = [vp]
        L.mt_last_error.argtypes = [vp]
        L.mt_last_error.restype = C.c_char_p
        L.mt_error_name.argtypes = [C.c_int]
        L.mt_error_name.restype = C.c_char_p
        L.mt_read_hidden.argtypes = [vp, i32, i32, vp, sz, vp]
        L.mt_profile_enable.argtypes = [vp, i32]
        L.mt_profile_read.argtypes = [vp, vp, vp]
        L.mt_share_weights.argtypes = [vp, vp]
        L.mt_schedule_steps.argtypes = [vp, vp]
        L.mt_debug_mfma_peak.argtypes = [i32, vp, C.c_size_t, vp, vp]
        L.mt_op_linear.argtypes = [i32, vp, i64, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, vp]
        L.mt_op_linear_batched.argtypes = [i32, i32, vp, i64, i64, vp, i64, vp, i64, vp, i64, vp, i64, i64, i32, i32, i32, i32, i32, vp]
        L.mt_op_attention.argtypes = [i32, vp, vp, vp, i32, i32, i32, i32, vp]
        L.mt_op_layernorm.argtypes = [vp, vp, vp, C.c_float, vp, vp, i32, i32, vp]
        L.mt_debug_set_gemm_tile.argtypes = [i32]
        L.mt_op_first_token_pool.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.mt_op_linear_sub.argtypes = [vp, i64, vp, i64, vp, vp, i64, i32, i32, i32, i32, i64, i64, i64, i64, vp, vp, i32, vp]
        L.mt_debug_set_gemm_tile.restype = i32
        _lib = L
    return _lib


class MTError(RuntimeError):
    def __init__(self, code, text=""):
        self.code = code
        name = lib().mt_error_name(code).decode()
        super().__init__(f"{name}: {text}" if text else name)


def make_config(spec, *, max_batch=None, max_seq=None, precision=None):
    """mt_config for an mt_synth.MTSpec-like object (fields vocab, hidden, ..., tasks)."""
    tasks = (mt_task_desc * len(spec.tasks))(*[mt_task_desc(t.fork_layer, t.n_layers, t.n_classes,
                                                            MT_HEAD_TOKEN if getattr(t, "token_level", False) else MT_HEAD_SEQUENCE)
                                               for t in spec.tasks])
    prec = precision if precision is not None else {"bf16": MT_BF16, "fp8": MT_FP8_FFN, "fp8_all": MT_FP8_LAYER}.get(spec.precision, MT_FP32_CHECK)
    cfg = mt_config(C.sizeof(mt_config), MT_ABI_VERSION, spec.vocab, spec.hidden, spec.heads, spec.ffn, spec.max_pos,
                    spec.type_vocab, spec.n_trunk_layers, len(spec.tasks), tasks, prec,
                    MT_GELU_TANH if spec.gelu == "tanh" else MT_GELU_ERF, spec.ln_eps,
                    spec.batch if max_batch is None else max_batch, spec.seq if max_seq is None else max_seq)
    cfg._keepalive = tasks
    return cfg


def pack_blob(scope: int, n_tensors: int, flat: np.ndarray) -> bytes:
    """Wrap a flat float32 parameter vector (canonical order) in the "MTW1" checkpoint header."""
    flat = np.ascontiguousarray(flat, dtype="<f4")
    return b"MTW1" + struct.pack("<iii", scope, n_tensors, 0) + flat.tobytes()


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Model:
    """Owns an mt_model plus the two torch-allocated arenas.  Methods mirror the C entry points."""

    def __init__(self, cfg: mt_config, device="cuda:0", bind=True):
        self.cfg = cfg
        self.h = C.c_void_p()
        rc = lib().mt_create(C.byref(cfg), C.byref(self.h))
        if rc != MT_OK:
            raise MTError(rc, "mt_create")
        self.device = device
        self.weights = self.workspace = None
        self.n_logits = lib().mt_n_logits(self.h)
        self.n_token_logits = lib().mt_n_token_logits(self.h)
        if bind:
            self.bind()

    def _check(self, rc):
        if rc != MT_OK:
            raise MTError(rc, lib().mt_last_error(self.h).decode())

    def close(self):
        if self.h:
            lib().mt_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def weight_bytes(self):
        return lib().mt_weight_bytes(self.h)

    def workspace_bytes(self):
        return lib().mt_workspace_bytes(self.h)

    def layer_count(self):
        return lib().mt_layer_count(self.h)

    def logit_offset(self, t):
        return lib().mt_logit_offset(self.h, t)

    def token_logit_offset(self, t):
        return lib().mt_token_logit_offset(self.h, t)

    def bind(self):
        import torch
        self.weights = torch.empty(self.weight_bytes(), dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(self.workspace_bytes(), dtype=torch.uint8, device=self.device)
        self._check(lib().mt_bind(self.h, _ptr(self.weights), self.weights.numel(), _ptr(self.workspace),
                                  self.workspace.numel()))

    def replica(self):
        """A second handle on the same weights with a workspace of its own (mt_share_weights): its forwards
        may overlap this model's on another stream."""
        import torch
        r = Model(self.cfg, device=self.device, bind=False)
        r.weights = self.weights
        r.workspace = torch.empty(r.workspace_bytes(), dtype=torch.uint8, device=self.device)
        r._check(lib().mt_bind(r.h, _ptr(r.weights), r.weights.numel(), _ptr(r.workspace), r.workspace.numel()))
        r._check(lib().mt_share_weights(r.h, self.h))
        return r

    def load_weights(self, scope: int, blob: bytes):
        buf = C.create_string_buffer(blob, len(blob)) if not isinstance(blob, C.Array) else blob
        self._check(lib().mt_load_weights(self.h, scope, C.cast(buf, C.c_void_p), len(blob), _stream()))

    def load_params(self, scope: int, flat: np.ndarray, n_tensors: int):
        self.load_weights(scope, pack_blob(scope, n_tensors, flat))

    def forward(self, ids, mask, out=None, task_mask=None, type_ids=None):
        """ids, mask (and optional segment ids type_ids): int32 CUDA tensors [B,S]; returns the float32 CUDA
        tensor [B, C_tot] (enqueued, not synced)."""
        import torch
        b, s = ids.shape
        if out is None:
            out = torch.zeros((b, self.n_logits), dtype=torch.float32, device=ids.device)
        tm = None
        if task_mask is not None:
            tm = (C.c_uint8 * len(task_mask))(*[1 if v else 0 for v in task_mask])
        if type_ids is None:
            self._check(lib().mt_forward(self.h, _ptr(ids), _ptr(mask), b, s, tm, _ptr(out), _stream()))
        else:
            assert type_ids.shape == ids.shape
            self._check(lib().mt_forward_typed(self.h, _ptr(ids), _ptr(type_ids), _ptr(mask), b, s, tm, _ptr(out), _stream()))
        return out

    def forward_multi(self, requests, outs=None, task_mask=None):
        """mt_forward_multi: `requests` is a list of (ids, mask) int32 CUDA tensor pairs of one shape [B,S]; returns the list
        of float32 CUDA tensors [B, C_tot], one per request (enqueued, not synced)."""
        import torch
        n = len(requests)
        b, s = requests[0][0].shape
        if outs is None:
            outs = [torch.zeros((b, self.n_logits), dtype=torch.float32, device=requests[0][0].device) for _ in range(n)]
        tm = None
        if task_mask is not None:
            tm = (C.c_uint8 * len(task_mask))(*[1 if v else 0 for v in task_mask])
        p_ids = (C.c_void_p * n)(*[r[0].data_ptr() for r in requests])
        p_mask = (C.c_void_p * n)(*[r[1].data_ptr() for r in requests])
        p_out = (C.c_void_p * n)(*[o.data_ptr() for o in outs])
        self._check(lib().mt_forward_multi(self.h, n, p_ids, p_mask, b, s, tm, p_out, _stream()))
        return outs

    def forward_requests(self, requests, outs=None, task_mask=None):
        """mt_forward_requests: `requests` is a list of (ids, mask) int32 CUDA tensor pairs [B_r, S] of one S and any B_r;
        returns the list of float32 CUDA tensors [B_r, C_tot], one per request (enqueued, not synced)."""
        import torch
        n = len(requests)
        s = requests[0][0].shape[1]
        sizes = [int(r[0].shape[0]) for r in requests]
        if outs is None:
            outs = [torch.zeros((b, self.n_logits), dtype=torch.float32, device=requests[0][0].device) for b in sizes]
        tm = None
        if task_mask is not None:
            tm = (C.c_uint8 * len(task_mask))(*[1 if v else 0 for v in task_mask])
        p_ids = (C.c_void_p * n)(*[r[0].data_ptr() for r in requests])
        p_mask = (C.c_void_p * n)(*[r[1].data_ptr() for r in requests])
        p_out = (C.c_void_p * n)(*[o.data_ptr() for o in outs])
        p_b = (C.c_int32 * n)(*sizes)
        self._check(lib().mt_forward_requests(self.h, n, p_ids, p_mask, p_b, s, tm, p_out, _stream()))
        return outs

    def forward_static(self, ids, mask, out, task_mask=None):
        """mt_forward_static: the forward pass on the library's fixed scratch array; `out` is the caller's float32
        CUDA tensor [B, C_tot] (this wrapper allocates nothing on the device either)."""
        b, s = ids.shape
        tm = None
        if task_mask is not None:
            tm = (C.c_uint8 * len(task_mask))(*[1 if v else 0 for v in task_mask])
        self._check(lib().mt_forward_static(self.h, _ptr(ids), _ptr(mask), b, s, tm, _ptr(out), _stream()))
        return out

    def forward_tokens(self, ids, mask, out=None, out_tokens=None, task_mask=None, type_ids=None):
        """mt_forward_tokens: returns (logits [B, C_tot], token logits [B, S, C_tok]), float32 CUDA tensors (enqueued,
        not synced)."""
        import torch
        b, s = ids.shape
        if out is None:
            out = torch.zeros((b, self.n_logits), dtype=torch.float32, device=ids.device)
        if out_tokens is None:
            out_tokens = torch.zeros((b, s, self.n_token_logits), dtype=torch.float32, device=ids.device)
        tm = None
        if task_mask is not None:
            tm = (C.c_uint8 * len(task_mask))(*[1 if v else 0 for v in task_mask])
        self._check(lib().mt_forward_tokens(self.h, _ptr(ids), _ptr(type_ids) if type_ids is not None else None, _ptr(mask), b, s, tm,
                                            _ptr(out) if out.numel() else None, _ptr(out_tokens) if out_tokens.numel() else None,
                                            _stream()))
        return out, out_tokens

    def forward_routed(self, ids, mask, route, out, type_ids=None):
        """route: [B][n_tasks] array-like of 0/1 (host); logits of wanted (b, t) pairs are written into `out`."""
        b, s = ids.shape
        r = np.ascontiguousarray(np.asarray(route) != 0, dtype=np.uint8)
        assert r.shape == (b, self.cfg.n_tasks)
        self._check(lib().mt_forward_routed(self.h, _ptr(ids), _ptr(type_ids) if type_ids is not None else None, _ptr(mask), b, s,
                                            r.ctypes.data_as(C.c_void_p), _ptr(out), _stream()))
        return out

    def forward_routed_tokens(self, ids, mask, route, out, out_tokens, type_ids=None):
        """mt_forward_routed_tokens: as forward_routed, token-level tasks' logits of wanted pairs go into `out_tokens`."""
        b, s = ids.shape
        r = np.ascontiguousarray(np.asarray(route) != 0, dtype=np.uint8)
        assert r.shape == (b, self.cfg.n_tasks)
        self._check(lib().mt_forward_routed_tokens(self.h, _ptr(ids), _ptr(type_ids) if type_ids is not None else None, _ptr(mask), b, s,
                                                   r.ctypes.data_as(C.c_void_p), _ptr(out) if out is not None and out.numel() else None,
                                                   _ptr(out_tokens) if out_tokens is not None and out_tokens.numel() else None, _stream()))
        return out, out_tokens

    def check_mask(self, mask):
        """mt_check_mask: number of sequences whose position 0 is padding (waits for the device); raises if any."""
        n = C.c_int32(-1)
        b, s = mask.shape
        rc = lib().mt_check_mask(self.h, _ptr(mask), b, s, C.byref(n), _stream())
        if rc != MT_OK:
            raise MTError(rc, lib().mt_last_error(self.h).decode())
        return int(n.value)

    def read_hidden(self, task: int, layer: int, batch: int, seq: int):
        import torch
        out = torch.empty((batch, seq, self.cfg.hidden), dtype=torch.float32, device=self.device)
        self._check(lib().mt_read_hidden(self.h, task, layer, _ptr(out), out.numel() * 4, _stream()))
        return out

    def profile_enable(self, on: bool):
        self._check(lib().mt_profile_enable(self.h, 1 if on else 0))

    def profile_read(self):
        ms = (C.c_float * len(KERNEL_CLASSES))()
        n = (C.c_int32 * len(KERNEL_CLASSES))()
        self._check(lib().mt_profile_read(self.h, ms, n))
        return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(KERNEL_CLASSES)}


def op_linear_sub(A, lda, W, ldw, bias, C, ldc, M, N, K, n_sub, sub_a, sub_w, sub_c, sub_bias=0, row0=None, rows=None,
                  out_f32=False):
    """mt_op_linear_sub on device tensors (raw strides and offsets in elements; C is written in place)."""
    rc = lib().mt_op_linear_sub(_ptr(A), lda, _ptr(W), ldw, _ptr(bias) if bias is not None else None, _ptr(C), ldc, M, N, K,
                                n_sub, sub_a, sub_w, sub_c, sub_bias, _ptr(row0) if row0 is not None else None,
                                _ptr(rows) if rows is not None else None, 1 if out_f32 else 0, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_linear_sub")
    return C


def op_first_token_pool(scores, x, seq_start, seq_len, batch, seq, hidden, heads, heads_pad):
    """mt_op_first_token_pool on device tensors; returns xbar [batch][heads_pad][hidden] bf16 (pad heads zero)."""
    import torch
    xbar = torch.zeros((batch, heads_pad, hidden), dtype=torch.bfloat16, device=x.device)
    rc = lib().mt_op_first_token_pool(_ptr(scores), _ptr(x), _ptr(xbar), _ptr(seq_start), _ptr(seq_len), batch, seq, hidden, heads,
                                      heads_pad, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_first_token_pool")
    return xbar


def mfma_peak(iters=4000):
    """Measured register-only bf16 matrix-core rate of the current device in TFLOP/s (mt_debug_mfma_peak)."""
    import torch
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = C.c_float(0.0)
    rc = lib().mt_debug_mfma_peak(iters, _ptr(scratch), scratch.numel(), C.byref(out), _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_debug_mfma_peak")
    return float(out.value)


def op_linear(precision, A, W, bias=None, residual=None, act=0, out_f32=False, lda=None):
    """C = act(A W^T + bias) (+ residual) on device tensors; A/W bf16 (MT_BF16) or float32 (MT_FP32_CHECK)."""
    import torch
    m, k = A.shape
    n = W.shape[0]
    dt = torch.float32 if (out_f32 or precision == MT_FP32_CHECK) else torch.bfloat16
    out = torch.empty((m, n), dtype=dt, device=A.device)
    rc = lib().mt_op_linear(precision, _ptr(A), A.stride(0) if lda is None else lda, _ptr(W), _ptr(bias), _ptr(residual),
                            _ptr(out), n, m, n, k, act, 1 if out_f32 else 0, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_linear")
    return out


def op_linear_batched(precision, A, W, bias=None, residual=None, act=0, out_f32=False, out=None):
    """Grouped form: A [G,M,K] (or [M,K], shared by all problems), W [G,N,K], bias [G,N], residual [G,M,N] -> C [G,M,N]."""
    import torch
    g, n, k = W.shape
    shared = A.dim() == 2
    m = A.shape[-2]
    dt = torch.float32 if (out_f32 or precision == MT_FP32_CHECK) else torch.bfloat16
    if out is None:
        out = torch.empty((g, m, n), dtype=dt, device=W.device)
    rc = lib().mt_op_linear_batched(precision, g, _ptr(A), 0 if shared else m * k, k, _ptr(W), n * k, _ptr(bias), n,
                                    _ptr(residual), m * n, _ptr(out), m * n, n, m, n, k, act, 1 if out_f32 else 0, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_linear_batched")
    return out


def e4m3_quantize(w):
    """(scale, uint8 codes) of a float32 array under the loader's FP8 storage rule (mt_debug_e4m3_quantize, host only)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    out = np.empty(w.size, dtype=np.uint8)
    s = lib().mt_debug_e4m3_quantize(w.ctypes.data_as(C.c_void_p), w.size, out.ctypes.data_as(C.c_void_p))
    return float(s), out.reshape(w.shape)


def op_linear_fp8(A, W, scale, bias=None, residual=None, act=0, out_kind=1, out_scale=1.0):
    """mt_op_linear_fp8 on device tensors: A [M,K], W [N,K] uint8 (E4M3 codes); returns C [M,N] (bf16 / float32 / uint8)."""
    import torch
    m, k = A.shape
    n = W.shape[0]
    dt = {0: torch.bfloat16, 1: torch.float32, 2: torch.uint8}[out_kind]
    out = torch.empty((m, n), dtype=dt, device=A.device)
    rc = lib().mt_op_linear_fp8(_ptr(A), k, _ptr(W), scale, _ptr(bias), _ptr(residual), _ptr(out), n, m, n, k, act, out_kind,
                                out_scale, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_linear_fp8")
    return out


def op_attention(precision, qkv, mask, batch, seq, hidden, heads):
    import torch
    ctx = torch.zeros((batch * seq, hidden), dtype=qkv.dtype, device=qkv.device)
    rc = lib().mt_op_attention(precision, _ptr(qkv), _ptr(mask), _ptr(ctx), batch, seq, hidden, heads, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_attention")
    return ctx


def op_layernorm(x, gamma, beta, eps, want_bf16=False):
    import torch
    m, h = x.shape
    of = torch.empty_like(x)
    ob = torch.empty((m, h), dtype=torch.bfloat16, device=x.device) if want_bf16 else None
    rc = lib().mt_op_layernorm(_ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(of), _ptr(ob), m, h, _stream())
    if rc != MT_OK:
        raise MTError(rc, "mt_op_layernorm")
    return (of, ob) if want_bf16 else of


def set_gemm_tile(sel: int) -> int:
    """Tuning aid: force one bf16 GEMM tile configuration (0 = choose by shape).  Returns the previous value."""
    return lib().mt_debug_set_gemm_tile(sel)
