"""ctypes wrapper around oracle/libwgkv_oracle.so (argument marshalling only).

TEST INFRASTRUCTURE: slow fp64 reference written from the paper; see
wgkv_oracle.c.  Arrays go in and out as numpy; K/V/Q are float32 arrays holding
the exact widening of the bf16 or fp32 inputs.
"""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None


class _CConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("w_local", C.c_int32),
                ("max_seqs", C.c_int32), ("max_global_pages", C.c_int32),
                ("n_pages", C.c_int64), ("keep_payload", C.c_int32)]


@dataclass
class OracleConfig:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_size: int
    w_local: int
    max_seqs: int
    max_global_pages: int
    n_pages: int
    keep_payload: bool = True


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("WGKV_ORACLE_LIB")  # e.g. the build with the sanitizers (see build.py)
        if path:
            path = os.path.abspath(path)
            if not os.path.exists(path):
                raise FileNotFoundError(f"WGKV_ORACLE_LIB names {path}, which does not exist")
        else:
            path = _build.LIB
            if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
                _build.build(force=True)
        L = C.CDLL(path)
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.POINTER(_CConfig)]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_push_tokens.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int32),
                                      C.POINTER(C.c_int32), C.POINTER(C.c_float),
                                      C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_float,
                                      C.POINTER(C.c_uint8), C.POINTER(C.c_uint8)]
        L.orc_free_seq.argtypes = [C.c_void_p, C.c_int]
        L.orc_seq_len.restype = C.c_int64
        L.orc_seq_len.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.orc_global_len.restype = C.c_int64
        L.orc_global_len.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        L.orc_free_top.restype = C.c_int64
        L.orc_free_top.argtypes = [C.c_void_p]
        L.orc_get_free_stack.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.orc_get_head_tables.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int,
                                          C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                          C.POINTER(C.c_float), C.POINTER(C.c_int64)]
        L.orc_get_global_pos.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int64)]
        L.orc_get_payload.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int] + [C.POINTER(C.c_float)] * 4
        L.orc_attend_cached.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_float),
                                        C.c_double, C.POINTER(C.c_double)]
        L.orc_attend_cached_batch.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int32),
                                              C.POINTER(C.c_float), C.c_double,
                                              C.POINTER(C.c_double), C.POINTER(C.c_int)]
        L.orc_attend_definition.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
                                            C.c_double, C.c_int64, C.POINTER(C.c_float),
                                            C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_int64,
                                            C.POINTER(C.c_float), C.POINTER(C.c_int64),
                                            C.POINTER(C.c_double)]
        L.orc_attend_soft.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int64,
                                      C.POINTER(C.c_float), C.POINTER(C.c_float),
                                      C.POINTER(C.c_float), C.c_int64, C.POINTER(C.c_float),
                                      C.POINTER(C.c_int64), C.c_int, C.c_double,
                                      C.POINTER(C.c_double)]
        fp, dp = C.POINTER(C.c_float), C.POINTER(C.c_double)
        L.orc_soft_attn_forward.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_double,
                                            fp, fp, fp, fp, dp, dp]
        L.orc_soft_attn_backward.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_double,
                                             fp, fp, fp, fp, fp, dp, dp, dp, dp]
        L.orc_sparsity_loss.argtypes = [C.c_int64, fp, dp, dp]
        L.orc_soft_attn_backward_sampled.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_double,
                                                     fp, fp, fp, fp, fp, C.c_int64, C.POINTER(C.c_int64), dp,
                                                     C.c_int, C.c_int64, dp, dp, dp]
        L.orc_linear_gate.argtypes = [C.c_int64, C.c_int, C.c_int, C.POINTER(C.c_float),
                                      C.POINTER(C.c_float), C.POINTER(C.c_double),
                                      C.POINTER(C.c_double)]
        L.orc_evict_scores.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), C.c_int,
                                       C.c_double, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.orc_evict_apply.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_float),
                                      C.c_int64, C.c_float, C.POINTER(C.c_int64)]
        L.orc_quest_page_scores.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float),
                                            C.POINTER(C.c_double)]
        L.orc_quest_select.argtypes = [C.POINTER(C.c_float), C.c_int64, C.c_int64, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_int32)]
        L.orc_attend_selected.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int32), C.c_int64, C.c_double, C.POINTER(C.c_double)]
        L.orc_gate_mlp.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int] + [C.POINTER(C.c_float)] * 6 + \
                                  [C.c_double, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        names = {-1: "bad argument", -2: "out of pages", -3: "page-table overflow", -4: "no memory"}
        super().__init__(f"oracle error {code} ({names.get(code, '?')})")
        self.code = code


class Oracle:
    """Mechanism oracle: dual cache + page tables, simulated token by token."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self._L = lib()
        cc = _CConfig(cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.page_size,
                      cfg.w_local, cfg.max_seqs, cfg.max_global_pages, cfg.n_pages,
                      1 if cfg.keep_payload else 0)
        self._s = self._L.orc_create(C.byref(cc))
        if not self._s:
            raise OracleError(-1)
        self.n_local_pages = -(-cfg.w_local // cfg.page_size)

    def __del__(self):
        if getattr(self, "_s", None):
            self._L.orc_destroy(self._s)
            self._s = None

    def push_tokens(self, layer, seq_ids, n_tokens, k, v, g, tau):
        """Prefill chunk / decode step: returns (admit_mask, promoted) uint8 [sum T, Hkv]."""
        seq_ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        n_tokens = np.ascontiguousarray(n_tokens, dtype=np.int32)
        total = int(n_tokens.sum())
        Hk, d = self.cfg.n_kv_heads, self.cfg.head_dim
        g = _f32(g).reshape(total, Hk)
        k = _f32(k)
        v = _f32(v)
        if k is not None:
            assert k.size == total * Hk * d and v.size == total * Hk * d
        admit = np.zeros((total, Hk), dtype=np.uint8)
        prom = np.zeros((total, Hk), dtype=np.uint8)
        rc = self._L.orc_push_tokens(self._s, layer, len(seq_ids), _p(seq_ids, C.c_int32),
                                     _p(n_tokens, C.c_int32), _p(k, C.c_float), _p(v, C.c_float),
                                     _p(g, C.c_float), np.float32(tau), _p(admit, C.c_uint8),
                                     _p(prom, C.c_uint8))
        if rc:
            raise OracleError(rc)
        return admit, prom

    def free_seq(self, seq):
        rc = self._L.orc_free_seq(self._s, seq)
        if rc:
            raise OracleError(rc)

    def seq_len(self, seq, layer):
        return int(self._L.orc_seq_len(self._s, seq, layer))

    def global_len(self, seq, layer, h):
        return int(self._L.orc_global_len(self._s, seq, layer, h))

    @property
    def free_top(self):
        return int(self._L.orc_free_top(self._s))

    def free_stack(self):
        out = np.zeros(max(self.cfg.n_pages, 1), dtype=np.int32)
        self._L.orc_get_free_stack(self._s, _p(out, C.c_int32))
        return out[: self.cfg.n_pages]

    def head_tables(self, seq, layer, h):
        """(local_pt, global_pt, ring_g, ring_pos) of one (seq, layer, kv head)."""
        lp = np.zeros(self.n_local_pages, dtype=np.int32)
        gp = np.zeros(max(self.cfg.max_global_pages, 1), dtype=np.int32)
        rg = np.zeros(self.cfg.w_local, dtype=np.float32)
        rp = np.zeros(self.cfg.w_local, dtype=np.int64)
        self._L.orc_get_head_tables(self._s, seq, layer, h, _p(lp, C.c_int32), _p(gp, C.c_int32),
                                    _p(rg, C.c_float), _p(rp, C.c_int64))
        return lp, gp[: self.cfg.max_global_pages], rg, rp

    def global_pos(self, seq, layer, h):
        n = self.global_len(seq, layer, h)
        out = np.zeros(max(n, 1), dtype=np.int64)
        self._L.orc_get_global_pos(self._s, seq, layer, h, _p(out, C.c_int64))
        return out[:n]

    def payload(self, seq, layer, h):
        """(global_k, global_v, ring_k, ring_v) float32 rows kept for this head."""
        n = self.global_len(seq, layer, h)
        d, W = self.cfg.head_dim, self.cfg.w_local
        gk = np.zeros((max(n, 1), d), dtype=np.float32)
        gv = np.zeros((max(n, 1), d), dtype=np.float32)
        rk = np.zeros((W, d), dtype=np.float32)
        rv = np.zeros((W, d), dtype=np.float32)
        rc = self._L.orc_get_payload(self._s, seq, layer, h, _p(gk, C.c_float), _p(gv, C.c_float),
                                     _p(rk, C.c_float), _p(rv, C.c_float))
        if rc:
            raise OracleError(rc)
        return gk[:n], gv[:n], rk, rv

    def evict_scores(self, layer, seq, h, q_obs, scale, pool_w=5):
        """(s_raw, s) importance of the entries of one head's global cache from the observation
        queries q_obs [n_obs, n_q_heads, d] (appendix "Eviction policy implementation")."""
        q_obs = _f32(q_obs)
        n_obs = q_obs.shape[0]
        assert q_obs.shape == (n_obs, self.cfg.n_q_heads, self.cfg.head_dim)
        n = self.global_len(seq, layer, h)
        raw = np.zeros(max(n, 1), dtype=np.float64)
        sm = np.zeros(max(n, 1), dtype=np.float64)
        rc = self._L.orc_evict_scores(self._s, layer, seq, h, _p(q_obs, C.c_float), n_obs, float(scale),
                                      int(pool_w), _p(raw, C.c_double), _p(sm, C.c_double))
        if rc:
            raise OracleError(rc)
        return raw[:n], sm[:n]

    def evict_apply(self, layer, seq_ids, scores, frac):
        """Removes the floor(frac * N) lowest-scored global entries of every head of the sequences;
        scores float32 [len(seq_ids) * n_kv_heads, stride].  Returns the number removed per unit."""
        seq_ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        scores = _f32(scores)
        n_units = len(seq_ids) * self.cfg.n_kv_heads
        assert scores.ndim == 2 and scores.shape[0] == n_units
        gone = np.zeros(max(n_units, 1), dtype=np.int64)
        rc = self._L.orc_evict_apply(self._s, layer, len(seq_ids), _p(seq_ids, C.c_int32), _p(scores, C.c_float),
                                     scores.shape[1], np.float32(frac), _p(gone, C.c_int64))
        if rc:
            raise OracleError(rc)
        return gone[:n_units]

    def quest_page_scores(self, layer, seq, h, q):
        """Criticality of every page of one head's global cache for the decode queries q [n_q_heads, d]."""
        q = _f32(q).reshape(self.cfg.n_q_heads, self.cfg.head_dim)
        n_pages = -(-self.global_len(seq, layer, h) // self.cfg.page_size)
        u = np.zeros(max(n_pages, 1), dtype=np.float64)
        rc = self._L.orc_quest_page_scores(self._s, layer, seq, h, _p(q, C.c_float), _p(u, C.c_double))
        if rc:
            raise OracleError(rc)
        return u[:n_pages]

    def attend_selected(self, seq, layer, q, sel, n_sel, scale):
        """Attention over the window and the selected pages; sel int32 [n_kv_heads, stride], n_sel [n_kv_heads]."""
        q = _f32(q).reshape(self.cfg.n_q_heads, self.cfg.head_dim)
        sel = np.ascontiguousarray(sel, dtype=np.int32)
        n_sel = np.ascontiguousarray(n_sel, dtype=np.int32)
        assert sel.ndim == 2 and sel.shape[0] == self.cfg.n_kv_heads == len(n_sel)
        out = np.zeros((self.cfg.n_q_heads, self.cfg.head_dim), dtype=np.float64)
        rc = self._L.orc_attend_selected(self._s, seq, layer, _p(q, C.c_float), _p(sel, C.c_int32), _p(n_sel, C.c_int32),
                                         sel.shape[1], float(scale), _p(out, C.c_double))
        if rc:
            raise OracleError(rc)
        return out

    def attend_cached(self, seq, layer, q, scale):
        q = _f32(q).reshape(self.cfg.n_q_heads, self.cfg.head_dim)
        out = np.zeros((self.cfg.n_q_heads, self.cfg.head_dim), dtype=np.float64)
        rc = self._L.orc_attend_cached(self._s, seq, layer, _p(q, C.c_float), float(scale),
                                       _p(out, C.c_double))
        if rc:
            raise OracleError(rc)
        return out

    def attend_cached_batch(self, layer, seq_ids, q, scale):
        """One decode step of one layer for several sequences; returns (out, threads)."""
        seq_ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        n = len(seq_ids)
        q = _f32(q).reshape(n, self.cfg.n_q_heads, self.cfg.head_dim)
        out = np.zeros(q.shape, dtype=np.float64)
        thr = C.c_int(0)
        rc = self._L.orc_attend_cached_batch(self._s, layer, n, _p(seq_ids, C.c_int32),
                                             _p(q, C.c_float), float(scale), _p(out, C.c_double),
                                             C.byref(thr))
        if rc:
            raise OracleError(rc)
        return out, thr.value


def attend_definition(K, V, g, q, q_pos, w_local, tau, scale):
    """Definition attention from the full history of one sequence/layer.

    K, V: [n_hist, Hkv, d]; g: [n_hist, Hkv]; q: [n_q, Hq, d]; q_pos: [n_q].
    """
    K = _f32(K); V = _f32(V); g = _f32(g); q = _f32(q)
    n_hist, Hk, d = K.shape
    n_q, Hq, _ = q.shape
    q_pos = np.ascontiguousarray(q_pos, dtype=np.int64)
    out = np.zeros((n_q, Hq, d), dtype=np.float64)
    rc = lib().orc_attend_definition(Hq, Hk, d, int(w_local), np.float32(tau), float(scale),
                                     n_hist, _p(K, C.c_float), _p(V, C.c_float), _p(g, C.c_float),
                                     n_q, _p(q, C.c_float), _p(q_pos, C.c_int64),
                                     _p(out, C.c_double))
    if rc:
        raise OracleError(rc)
    return out


def attend_soft(K, V, g, q, q_pos, w_local, scale, use_log=False, eps=0.0):
    K = _f32(K); V = _f32(V); g = _f32(g); q = _f32(q)
    n_hist, Hk, d = K.shape
    n_q, Hq, _ = q.shape
    q_pos = np.ascontiguousarray(q_pos, dtype=np.int64)
    out = np.zeros((n_q, Hq, d), dtype=np.float64)
    rc = lib().orc_attend_soft(Hq, Hk, d, int(w_local), float(scale), n_hist, _p(K, C.c_float),
                               _p(V, C.c_float), _p(g, C.c_float), n_q, _p(q, C.c_float),
                               _p(q_pos, C.c_int64), 1 if use_log else 0, float(eps),
                               _p(out, C.c_double))
    if rc:
        raise OracleError(rc)
    return out


def soft_attn_forward(Q, K, V, g, w_local, scale, eps):
    """Training-time Write-Gated Attention of one sequence (Sec. 3.2, log-space form):
    (out [T, Hq, d], lse [T, Hq]) in fp64 for Q [T, Hq, d], K, V [T, Hkv, d], g [T, Hkv]."""
    Q = _f32(Q); K = _f32(K); V = _f32(V); g = _f32(g)
    T, Hq, d = Q.shape
    Hk = K.shape[1]
    assert K.shape == (T, Hk, d) and V.shape == (T, Hk, d) and g.shape == (T, Hk)
    out = np.zeros((T, Hq, d), dtype=np.float64)
    lse = np.zeros((T, Hq), dtype=np.float64)
    rc = lib().orc_soft_attn_forward(T, Hq, Hk, d, int(w_local), float(scale), float(eps), _p(Q, C.c_float),
                                     _p(K, C.c_float), _p(V, C.c_float), _p(g, C.c_float),
                                     _p(out, C.c_double), _p(lse, C.c_double))
    if rc:
        raise OracleError(rc)
    return out, lse


def soft_attn_backward(Q, K, V, g, dO, w_local, scale, eps):
    """(dQ, dK, dV, dg) in fp64 of a loss with dLoss/dOut = dO through soft_attn_forward."""
    Q = _f32(Q); K = _f32(K); V = _f32(V); g = _f32(g); dO = _f32(dO)
    T, Hq, d = Q.shape
    Hk = K.shape[1]
    assert K.shape == (T, Hk, d) and V.shape == (T, Hk, d) and g.shape == (T, Hk) and dO.shape == Q.shape
    dQ = np.zeros((T, Hq, d), dtype=np.float64)
    dK = np.zeros((T, Hk, d), dtype=np.float64)
    dV = np.zeros((T, Hk, d), dtype=np.float64)
    dg = np.zeros((T, Hk), dtype=np.float64)
    rc = lib().orc_soft_attn_backward(T, Hq, Hk, d, int(w_local), float(scale), float(eps), _p(Q, C.c_float),
                                      _p(K, C.c_float), _p(V, C.c_float), _p(g, C.c_float), _p(dO, C.c_float),
                                      _p(dQ, C.c_double), _p(dK, C.c_double), _p(dV, C.c_double),
                                      _p(dg, C.c_double))
    if rc:
        raise OracleError(rc)
    return dQ, dK, dV, dg


def soft_attn_backward_sampled(Q, K, V, g, dO, w_local, scale, eps, rows, h, j_first):
    """The gradients of soft_attn_backward for a sample: dQ [len(rows), Hq, d] of the listed query rows, and
    (dK, dV [T - j_first, d], dg [T - j_first]) of the keys j >= j_first of kv head h."""
    Q = _f32(Q); K = _f32(K); V = _f32(V); g = _f32(g); dO = _f32(dO)
    T, Hq, d = Q.shape
    Hk = K.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n = T - int(j_first)
    dQ = np.zeros((len(rows), Hq, d), dtype=np.float64)
    dK = np.zeros((n, d), dtype=np.float64)
    dV = np.zeros((n, d), dtype=np.float64)
    dg = np.zeros((n,), dtype=np.float64)
    rc = lib().orc_soft_attn_backward_sampled(T, Hq, Hk, d, int(w_local), float(scale), float(eps), _p(Q, C.c_float),
                                              _p(K, C.c_float), _p(V, C.c_float), _p(g, C.c_float), _p(dO, C.c_float),
                                              len(rows), _p(rows, C.c_int64), _p(dQ, C.c_double), int(h), int(j_first),
                                              _p(dK, C.c_double), _p(dV, C.c_double), _p(dg, C.c_double))
    if rc:
        raise OracleError(rc)
    return dQ, dK, dV, dg


def sparsity_loss(g):
    """(loss, dloss/dg) of the sparsity term of the training objective (Sec. 3.3) over all scores."""
    g = _f32(g)
    loss = C.c_double(0.0)
    dg = np.zeros(g.shape, dtype=np.float64)
    rc = lib().orc_sparsity_loss(g.size, _p(g, C.c_float), C.byref(loss), _p(dg, C.c_double))
    if rc:
        raise OracleError(rc)
    return loss.value, dg


def linear_gate(hidden, w):
    """(logit, g) in fp64 for hidden [T, dim] and w [Hkv, dim]."""
    hidden = _f32(hidden); w = _f32(w)
    T, dim = hidden.shape
    Hk = w.shape[0]
    logit = np.zeros((T, Hk), dtype=np.float64)
    g = np.zeros((T, Hk), dtype=np.float64)
    lib().orc_linear_gate(T, dim, Hk, _p(hidden, C.c_float), _p(w, C.c_float),
                          _p(logit, C.c_double), _p(g, C.c_double))
    return logit, g


def gate_mlp(k, k_rope, W1, b1, W2, b2, eps=1e-6, feature_bf16=False):
    """(logit, g) in fp64 of the Write-Gate MLP (Sec. 3.2) for k, k_rope [T, Hkv, d],
    W1 [Hkv, width, 2d], b1 [Hkv, width], W2 [Hkv, width], b2 [Hkv]."""
    k = _f32(k); k_rope = _f32(k_rope); W1 = _f32(W1); b1 = _f32(b1); W2 = _f32(W2); b2 = _f32(b2)
    T, Hk, d = k.shape
    width = W1.shape[1]
    assert k_rope.shape == k.shape and W1.shape == (Hk, width, 2 * d)
    assert b1.shape == (Hk, width) and W2.shape == (Hk, width) and b2.shape == (Hk,)
    logit = np.zeros((T, Hk), dtype=np.float64)
    g = np.zeros((T, Hk), dtype=np.float64)
    rc = lib().orc_gate_mlp(T, Hk, d, width, _p(k, C.c_float), _p(k_rope, C.c_float), _p(W1, C.c_float),
                            _p(b1, C.c_float), _p(W2, C.c_float), _p(b2, C.c_float), C.c_double(eps),
                            1 if feature_bf16 else 0, _p(logit, C.c_double), _p(g, C.c_double))
    assert rc == 0, rc
    return logit, g


def quest_select(scores, budget_pages):
    """Ascending indices of the min(n_pages, budget_pages) pages with the largest fp32 scores
    (equal scores: lower index first)."""
    scores = _f32(scores).ravel()
    sel = np.zeros(max(budget_pages, 1), dtype=np.int32)
    n = C.c_int32(0)
    rc = lib().orc_quest_select(_p(scores, C.c_float), len(scores), int(budget_pages), _p(sel, C.c_int32), C.byref(n))
    assert rc == 0, rc
    return sel[: n.value].copy()
