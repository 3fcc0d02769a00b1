"""Thin ctypes binding of libtgnn.so.  Argument marshalling only: every step of the training path runs in
the HIP kernels behind the C ABI (include/tgnn.h).  PyTorch supplies device memory and streams.

The library must have been built (python -m paper_2307_07649_amd.build); importing this module raises if
libtgnn.so is missing -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_LIB_PATH = os.environ.get("TGNN_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtgnn.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} not found: build it with `python -m paper_2307_07649_amd.build`")
_lib = C.CDLL(_LIB_PATH)

PARAM_NAMES = ["time_w", "time_b", "gru_wih", "gru_whh", "gru_bih", "gru_bhh", "wq", "bq", "wk", "bk",
               "wv", "bv", "wo", "bo", "dec_ws", "dec_wd", "dec_b1", "dec_w2", "dec_b2"]
MAX_BATCHES = 16
MAX_STEPS_PER_CALL = 8
FLAG_OVERWRITE_GRADS = 1
FLAG_SIDE_STREAM = 2
FLAG_NO_GRAPH = 4
FLAG_WIDE_ROOT_TILES = 8
FLAG_GENERIC_ATTN = 16


class tgnn_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_nodes", "d_mem", "d_time", "d_edge", "d_static", "n_heads", "k",
                                         "max_batch", "n_replicas", "dt_source", "flags", "max_neg_sets",
                                         "n_classes")]


class tgnn_graph(C.Structure):
    _fields_ = [("indptr", C.c_void_p), ("nbr", C.c_void_p), ("eid", C.c_void_p), ("ts", C.c_void_p),
                ("efeat", C.c_void_p), ("n_events", C.c_int64)]


class tgnn_state(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("mem", "mem_ts", "mail", "mail_ts", "mail_eid", "stat")]


class tgnn_params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class tgnn_batch(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("neg", C.c_void_p), ("eid", C.c_void_p),
                ("t", C.c_void_p), ("n", C.c_int32), ("replica", C.c_int32)]


_P = C.c_void_p
_I = C.c_int32
_SIGS = {
    "tgnn_last_error": (C.c_char_p, []),
    "tgnn_create": (_I, [C.POINTER(tgnn_config), C.POINTER(_P)]),
    "tgnn_destroy": (_I, [_P]),
    "tgnn_workspace_bytes": (C.c_int64, [_P]),
    "tgnn_build_tcsr": (_I, [_P, _P, _P, C.c_int64, _I, _P, _P, _P, _P]),
    "tgnn_state_reset": (_I, [_P, C.POINTER(tgnn_state), _I, _P]),
    "tgnn_sample_recent": (_I, [_P, C.POINTER(tgnn_graph), _P, _P, _I, _P, _P, _P, _P, _P]),
    "tgnn_gather_memory": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), _I, _P, _I, _P, _P, _P, _P, _P, _P, _P]),
    "tgnn_gru_update": (_I, [_P, C.POINTER(tgnn_params), _I, _P, _P, _P, _P, _P, _P, _P, _P, _P]),
    "tgnn_temporal_attn_fwd": (_I, [_P, C.POINTER(tgnn_params), _I, _P, _P, _P, _P, _P, _P, _P]),
    "tgnn_temporal_attn_bwd": (_I, [_P, C.POINTER(tgnn_params), _I, _P, C.POINTER(tgnn_params), _P, _P, _P]),
    "tgnn_memory_writeback": (_I, [_P, C.POINTER(tgnn_state), _I, _P, _P, _P, _P, _I, _P, _P, _P, _P, _P, _P]),
    "tgnn_memory_writeback_noalloc": (_I, [_I, _I, C.POINTER(tgnn_state), _P, _P, _P, _P, _I, _P, _P, _P, _P, _P, _P]),
    "tgnn_train_step": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), C.POINTER(tgnn_params),
                             C.POINTER(tgnn_params), C.POINTER(tgnn_batch), _I, C.c_float, _P, _P, _P, _P]),
    "tgnn_train_step_epoch_parallel": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), C.POINTER(tgnn_params),
                                            C.POINTER(tgnn_params), C.POINTER(tgnn_batch), _I, _I, C.c_float, _P, _P, _P, _P]),
    "tgnn_train_step_edge_class": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), C.POINTER(tgnn_params),
                                        C.POINTER(tgnn_params), C.POINTER(tgnn_batch), _I, C.POINTER(_P), C.c_float, _P, _P,
                                        _P, _P]),
    "tgnn_eval_step": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), C.POINTER(tgnn_params), C.POINTER(tgnn_batch),
                            _I, _I, _P, _P, _P, _P, _P]),
    "tgnn_eval_step_edge_class": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), C.POINTER(tgnn_params),
                                       C.POINTER(tgnn_batch), _I, C.POINTER(_P), _P, _P, _P, _P]),
    "tgnn_train_steps": (_I, [_P, C.POINTER(tgnn_graph), C.POINTER(tgnn_state), C.POINTER(tgnn_params),
                              C.POINTER(tgnn_params), _I, C.POINTER(tgnn_batch), _I, C.c_float, _P, _P]),
    "tgnn_set_optimizer": (_I, [_P, _I, C.POINTER(tgnn_params), C.POINTER(tgnn_params), C.c_float, C.c_float, C.c_float]),
    "tgnn_train_static": (_I, [_P, _I, _P, C.c_float]),
    "tgnn_debug_read": (_I, [_P, _I, _P, C.c_int64, _P]),
    "tgnn_debug_copy": (_I, [_P, _P, C.c_int64, _P]),
    "tgnn_zero_params": (_I, [_P, C.POINTER(tgnn_params), _P]),
    "tgnn_profile_enable": (_I, [_P, C.c_uint32]),
    "tgnn_profile_every": (_I, [_P, _I]),
    "tgnn_profile_read": (_I, [_P, _I, C.POINTER(_I), C.POINTER(C.c_double)]),
}
EXPORTS = list(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)          # AttributeError here = the library does not export a declared symbol
    _fn.restype = _res
    _fn.argtypes = _args


class TgnnError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"libtgnn error {code}: {_lib.tgnn_last_error().decode()}")


def _check(rc):
    if rc != 0:
        raise TgnnError(rc)


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensor must be contiguous"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def build_tcsr(src, dst, ts, n_nodes):
    """HOST.  numpy int32/int32/float64 event list -> (indptr i64, nbr i32, eid i32, ts f64) numpy arrays."""
    src = np.ascontiguousarray(src, np.int32); dst = np.ascontiguousarray(dst, np.int32)
    ts = np.ascontiguousarray(ts, np.float64)
    E = len(src)
    indptr = np.empty(n_nodes + 1, np.int64); nbr = np.empty(2 * E, np.int32); eid = np.empty(2 * E, np.int32)
    tso = np.empty(2 * E, np.float64)
    _check(_lib.tgnn_build_tcsr(src.ctypes.data, dst.ctypes.data, ts.ctypes.data, E, n_nodes, indptr.ctypes.data,
                                nbr.ctypes.data, eid.ctypes.data, tso.ctypes.data))
    return indptr, nbr, eid, tso


def tgnn_debug_copy(dst, src):
    """dst[:] = src through the library's plain copy kernel (HBM-traffic counter calibration)."""
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    _check(_lib.tgnn_debug_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream()))


def tgnn_memory_writeback_noalloc(st, src, dst, eid, t, s_src, s_dst, tau_src, tau_dst, out_winner):
    """st: a State of one replica; out_winner: int32 device tensor [2 n] (preallocated by the caller: the call
    itself allocates nothing)."""
    n_nodes, d_mem = st.mem.shape
    _check(_lib.tgnn_memory_writeback_noalloc(n_nodes, d_mem, C.byref(st.c), _ptr(src), _ptr(dst), _ptr(eid), _ptr(t),
                                              src.numel(), _ptr(s_src), _ptr(s_dst), _ptr(tau_src), _ptr(tau_dst),
                                              _ptr(out_winner), _stream()))
    return out_winner


class Graph:
    """Device-resident temporal CSR + edge features."""

    def __init__(self, src, dst, ts, n_nodes, efeat, device="cuda"):
        indptr, nbr, eid, tso = build_tcsr(src, dst, ts, n_nodes)
        self.n_events = len(src)
        self.indptr = torch.from_numpy(indptr).to(device)
        self.nbr = torch.from_numpy(nbr).to(device)
        self.eid = torch.from_numpy(eid).to(device)
        self.ts = torch.from_numpy(tso).to(device)
        if efeat is None:
            self.efeat = None
        elif isinstance(efeat, torch.Tensor):
            self.efeat = efeat.to(device).contiguous()
        else:
            self.efeat = torch.from_numpy(np.ascontiguousarray(efeat, np.float32)).to(device)
        self.c = tgnn_graph(_ptr(self.indptr), _ptr(self.nbr), _ptr(self.eid), _ptr(self.ts), _ptr(self.efeat),
                            self.n_events)


class State:
    def __init__(self, n_nodes, d_mem, n_replicas=1, static=None, device="cuda"):
        n = n_nodes * n_replicas
        self.mem = torch.zeros(n, d_mem, dtype=torch.float32, device=device)
        self.mem_ts = torch.zeros(n, dtype=torch.float64, device=device)
        self.mail = torch.zeros(n, 2 * d_mem, dtype=torch.float32, device=device)
        self.mail_ts = torch.zeros(n, dtype=torch.float64, device=device)
        self.mail_eid = torch.full((n,), -1, dtype=torch.int32, device=device)
        self.stat = None if static is None else torch.as_tensor(static, dtype=torch.float32).to(device).contiguous()
        self.c = tgnn_state(_ptr(self.mem), _ptr(self.mem_ts), _ptr(self.mail), _ptr(self.mail_ts),
                            _ptr(self.mail_eid), _ptr(self.stat))


class Params:
    """Named float32 device tensors in the layout of tgnn_params."""

    def __init__(self, tensors: dict):
        self.t = {n: tensors[n].contiguous() for n in PARAM_NAMES}
        self.c = tgnn_params(*[_ptr(self.t[n]) for n in PARAM_NAMES])

    @classmethod
    def from_numpy(cls, arrays: dict, device="cuda"):
        return cls({n: torch.from_numpy(np.ascontiguousarray(arrays[n], np.float32)).to(device) for n in PARAM_NAMES})

    @classmethod
    def zeros_like(cls, other: "Params"):
        return cls({n: torch.zeros_like(other.t[n]) for n in PARAM_NAMES})

    def zero_(self):
        for v in self.t.values():
            v.zero_()

    def numpy(self):
        return {n: v.detach().cpu().numpy() for n, v in self.t.items()}


class Batch:
    def __init__(self, src, dst, neg, eid, t, replica=0, device="cuda"):
        def dev(a, dt):
            if isinstance(a, torch.Tensor):
                return a.to(device=device, dtype=dt).contiguous()
            return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dt)
        self.src, self.dst, self.neg, self.eid = (dev(a, torch.int32) for a in (src, dst, neg, eid))
        self.t = dev(t, torch.float64)
        self.n = int(self.src.numel())
        self.replica = replica
        self.c = tgnn_batch(_ptr(self.src), _ptr(self.dst), _ptr(self.neg), _ptr(self.eid), _ptr(self.t), self.n, replica)


class Context:
    def __init__(self, n_nodes, d_mem, d_time, d_edge, d_static, n_heads, k, max_batch, n_replicas=1, dt_source=0,
                 flags=0, max_neg_sets=1, n_classes=0):
        self.cfg = tgnn_config(n_nodes, d_mem, d_time, d_edge, d_static, n_heads, k, max_batch, n_replicas, dt_source,
                               flags, max_neg_sets, n_classes)
        self.h = _P()
        _check(_lib.tgnn_create(C.byref(self.cfg), C.byref(self.h)))
        self.d_x = d_mem + d_static

    def close(self):
        if self.h:
            _check(_lib.tgnn_destroy(self.h))
            self.h = _P()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def workspace_bytes(self):
        return _lib.tgnn_workspace_bytes(self.h)

    # ---- entry points (same names as the C ABI) ----
    def tgnn_state_reset(self, st: State, replica=-1):
        _check(_lib.tgnn_state_reset(self.h, C.byref(st.c), replica, _stream()))

    def tgnn_sample_recent(self, g: Graph, node, t):
        n, k = node.numel(), self.cfg.k
        dev = node.device
        nbr = torch.empty(n, k, dtype=torch.int32, device=dev); eid = torch.empty_like(nbr)
        ts = torch.empty(n, k, dtype=torch.float64, device=dev); cnt = torch.empty(n, dtype=torch.int32, device=dev)
        _check(_lib.tgnn_sample_recent(self.h, C.byref(g.c), _ptr(node), _ptr(t), n, _ptr(nbr), _ptr(eid), _ptr(ts),
                                       _ptr(cnt), _stream()))
        return nbr, eid, ts, cnt

    def tgnn_gather_memory(self, g: Graph, st: State, replica, slot_node, out=None):
        n = slot_node.numel(); dev = slot_node.device
        dm, de = self.cfg.d_mem, self.cfg.d_edge
        if out is None:
            out = dict(mem=torch.empty(n, dm, device=dev), mail=torch.empty(n, 2 * dm, device=dev),
                       mail_efeat=torch.empty(n, de, device=dev),
                       mem_ts=torch.empty(n, dtype=torch.float64, device=dev),
                       mail_ts=torch.empty(n, dtype=torch.float64, device=dev),
                       has_mail=torch.empty(n, dtype=torch.int32, device=dev))
        _check(_lib.tgnn_gather_memory(self.h, C.byref(g.c), C.byref(st.c), replica, _ptr(slot_node), n,
                                       _ptr(out["mem"]), _ptr(out["mail"]), _ptr(out["mail_efeat"]) if de else None,
                                       _ptr(out["mem_ts"]), _ptr(out["mail_ts"]), _ptr(out["has_mail"]), _stream()))
        return out

    def tgnn_gru_update(self, p: Params, staged: dict):
        n = staged["mem"].shape[0]; dev = staged["mem"].device
        s_new = torch.empty(n, self.cfg.d_mem, device=dev); tau = torch.empty(n, dtype=torch.float64, device=dev)
        _check(_lib.tgnn_gru_update(self.h, C.byref(p.c), n, _ptr(staged["mem"]), _ptr(staged["mail"]),
                                    _ptr(staged["mail_efeat"]) if self.cfg.d_edge else None, _ptr(staged["mem_ts"]),
                                    _ptr(staged["mail_ts"]), _ptr(staged["has_mail"]), _ptr(s_new), _ptr(tau), _stream()))
        return s_new, tau

    def tgnn_temporal_attn_fwd(self, p: Params, x_root, x_nbr, e_nbr, dt_nbr, cnt):
        R = x_root.shape[0]
        z = torch.empty(R, self.cfg.d_mem, device=x_root.device)
        _check(_lib.tgnn_temporal_attn_fwd(self.h, C.byref(p.c), R, _ptr(x_root), _ptr(x_nbr),
                                           _ptr(e_nbr) if self.cfg.d_edge else None, _ptr(dt_nbr), _ptr(cnt), _ptr(z),
                                           _stream()))
        return z

    def tgnn_temporal_attn_bwd(self, p: Params, dz, grads: Params):
        R = dz.shape[0]; dm = self.cfg.d_mem
        d_root = torch.empty(R, dm, device=dz.device); d_nbr = torch.empty(R * self.cfg.k, dm, device=dz.device)
        _check(_lib.tgnn_temporal_attn_bwd(self.h, C.byref(p.c), R, _ptr(dz), C.byref(grads.c), _ptr(d_root),
                                           _ptr(d_nbr), _stream()))
        return d_root, d_nbr

    def tgnn_memory_writeback(self, st: State, replica, src, dst, eid, t, s_src, s_dst, tau_src, tau_dst):
        n = src.numel()
        win = torch.empty(2 * n, dtype=torch.int32, device=src.device)
        _check(_lib.tgnn_memory_writeback(self.h, C.byref(st.c), replica, _ptr(src), _ptr(dst), _ptr(eid), _ptr(t), n,
                                          _ptr(s_src), _ptr(s_dst), _ptr(tau_src), _ptr(tau_dst), _ptr(win), _stream()))
        return win

    def tgnn_train_step(self, g: Graph, st: State, p: Params, grads: Params, batches, lr=0.0, out_loss=None,
                        out_logits=None, out_winner=None):
        arr = (tgnn_batch * len(batches))(*[b.c for b in batches])
        _check(_lib.tgnn_train_step(self.h, C.byref(g.c), C.byref(st.c), C.byref(p.c), C.byref(grads.c), arr,
                                    len(batches), lr, _ptr(out_loss), _ptr(out_logits), _ptr(out_winner), _stream()))

    def tgnn_train_step_epoch_parallel(self, g: Graph, st: State, p: Params, grads: Params, batches, n_neg_sets, lr=0.0,
                                       out_loss=None, out_logits=None, out_winner=None):
        """Each batch's `neg` holds n_neg_sets sets of n negative destinations, one after the other."""
        arr = (tgnn_batch * len(batches))(*[b.c for b in batches])
        _check(_lib.tgnn_train_step_epoch_parallel(self.h, C.byref(g.c), C.byref(st.c), C.byref(p.c), C.byref(grads.c), arr,
                                                   len(batches), n_neg_sets, lr, _ptr(out_loss), _ptr(out_logits),
                                                   _ptr(out_winner), _stream()))

    def tgnn_train_step_edge_class(self, g: Graph, st: State, p: Params, grads: Params, batches, labels, lr=0.0,
                                   out_loss=None, out_logits=None, out_winner=None):
        """labels: one float32 device tensor [n, n_classes] per batch (the batches' `neg` is not read)."""
        arr = (tgnn_batch * len(batches))(*[b.c for b in batches])
        lab = (_P * len(batches))(*[_ptr(y) for y in labels])
        _check(_lib.tgnn_train_step_edge_class(self.h, C.byref(g.c), C.byref(st.c), C.byref(p.c), C.byref(grads.c), arr,
                                               len(batches), lab, lr, _ptr(out_loss), _ptr(out_logits), _ptr(out_winner),
                                               _stream()))

    def tgnn_eval_step(self, g: Graph, st: State, p: Params, batches, n_neg_sets, out_rank, out_rr_sum, out_logits=None,
                       out_winner=None):
        """Each batch's `neg` holds n_neg_sets sets of n negative destinations; out_rank [sum n] float32, out_rr_sum [1]
        float32 (the sum of 1 / rank is added to it)."""
        arr = (tgnn_batch * len(batches))(*[b.c for b in batches])
        _check(_lib.tgnn_eval_step(self.h, C.byref(g.c), C.byref(st.c), C.byref(p.c), arr, len(batches), n_neg_sets,
                                   _ptr(out_logits), _ptr(out_rank), _ptr(out_rr_sum), _ptr(out_winner), _stream()))

    def tgnn_eval_step_edge_class(self, g: Graph, st: State, p: Params, batches, labels, out_counts, out_logits=None,
                                  out_winner=None):
        """labels: one float32 device tensor [n, n_classes] per batch; out_counts: int32 device tensor [3], the counts
        tp, fp, fn of the predictions logit > 0 are added to it."""
        arr = (tgnn_batch * len(batches))(*[b.c for b in batches])
        lab = (_P * len(batches))(*[_ptr(y) for y in labels])
        _check(_lib.tgnn_eval_step_edge_class(self.h, C.byref(g.c), C.byref(st.c), C.byref(p.c), arr, len(batches), lab,
                                              _ptr(out_logits), _ptr(out_counts), _ptr(out_winner), _stream()))

    def tgnn_train_steps(self, g: Graph, st: State, p: Params, grads: Params, steps, lr=0.0, out_loss=None):
        """steps: a list of steps, each a list of Batch (the same number per step); out_loss: device array [len(steps)]."""
        nb = len(steps[0])
        flat = [b.c for step in steps for b in step]
        arr = (tgnn_batch * len(flat))(*flat)
        _check(_lib.tgnn_train_steps(self.h, C.byref(g.c), C.byref(st.c), C.byref(p.c), C.byref(grads.c), len(steps), arr,
                                     nb, lr, _ptr(out_loss), _stream()))

    def tgnn_set_optimizer(self, kind, m: Params = None, v: Params = None, beta1=0.9, beta2=0.999, eps=1e-8):
        self._opt = (m, v)      # keeps the moment tensors alive
        _check(_lib.tgnn_set_optimizer(self.h, kind, C.byref(m.c) if m else None, C.byref(v.c) if v else None, beta1, beta2,
                                       eps))

    def tgnn_train_static(self, enable, grad_static=None, lr_static=0.0):
        self._gstat = grad_static
        _check(_lib.tgnn_train_static(self.h, 1 if enable else 0, _ptr(grad_static), lr_static))

    def tgnn_zero_params(self, grads: Params):
        _check(_lib.tgnn_zero_params(self.h, C.byref(grads.c), _stream()))

    def tgnn_profile_enable(self, stage_mask: int):
        _check(_lib.tgnn_profile_enable(self.h, stage_mask))

    def tgnn_profile_every(self, n: int):
        _check(_lib.tgnn_profile_every(self.h, n))

    def tgnn_profile_read(self, stage: int):
        cnt = _I(0); ms = C.c_double(0.0)
        _check(_lib.tgnn_profile_read(self.h, stage, C.byref(cnt), C.byref(ms)))
        return cnt.value, ms.value

    def tgnn_debug_read(self, what, dst):
        _check(_lib.tgnn_debug_read(self.h, what, _ptr(dst), dst.numel() * dst.element_size(), _stream()))
        return dst
