"""ctypes binding with the same names as the C ABI (include/wgkv.h).

Argument marshalling only.  Tensors are torch CUDA tensors; small per-call
arrays are Python sequences.  Every call enqueues on torch's current stream.
"""
import ctypes as C
import os
from dataclasses import dataclass

F32, BF16 = 0, 1

EXPORTED_SYMBOLS = [
    "wgkv_version", "wgkv_get_meta_layout", "wgkv_query_sizes", "wgkv_init_pool",
    "wgkv_gate_scores", "wgkv_gate_mlp_scores", "wgkv_prefill_admit", "wgkv_prefill_admit_bounded", "wgkv_decode_step", "wgkv_decode_promote", "wgkv_attend", "wgkv_attend_decode_static", "wgkv_tune_decode_attention", "wgkv_evict_scores", "wgkv_evict_apply", "wgkv_quest_landmark_bytes", "wgkv_quest_update",
    "wgkv_quest_select", "wgkv_attend_selected", "wgkv_soft_attn_forward", "wgkv_soft_attn_workspace_bytes",
    "wgkv_soft_attn_backward", "wgkv_sparsity_loss", "wgkv_free_seq",
    "wgkv_status", "wgkv_clear_error", "wgkv_stream_read_probe", "wgkv_set_profile_events", "wgkv_destroy",
]

_ERR = {-1: "invalid argument", -2: "out of pages", -3: "page-table overflow", -4: "HIP error",
        -5: "device error flag set", -6: "workspace too small", -7: "host out of memory",
        -8: "a head admitted more tokens than the bound given to wgkv_prefill_admit_bounded",
        -9: "a decode step relied on wgkv_decode_promote, which had not handled this token"}


class WgkvError(RuntimeError):
    def __init__(self, code, what=""):
        super().__init__(f"{what}: wgkv error {code} ({_ERR.get(code, '?')})")
        self.code = code


class _CConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("page_size", C.c_int32),
                ("w_local", C.c_int32), ("max_seqs", C.c_int32),
                ("max_global_pages_per_head", C.c_int32), ("n_pages", C.c_int64)]


class _CLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("seq_len", "global_len", "local_pt", "global_pt", "ring_g",
                                          "free_stack", "free_top", "err_flag", "unit_counters", "ahead",
                                          "total_bytes")] + \
               [("n_local_pages", C.c_int32)]


@dataclass
class Config:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    page_size: int
    w_local: int
    max_seqs: int
    max_global_pages_per_head: int
    n_pages: int

    def c(self):
        return _CConfig(self.n_layers, self.n_q_heads, self.n_kv_heads, self.head_dim, self.dtype,
                        self.page_size, self.w_local, self.max_seqs,
                        self.max_global_pages_per_head, self.n_pages)


def library_path() -> str:
    override = os.environ.get("WGKV_LIB")   # e.g. the build with a sanitized host side (see build.py)
    if override:
        return os.path.abspath(override)
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libwgkv.so")


_lib = None


def load_library():
    """Load the built C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2512_17452_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    pi32 = C.POINTER(C.c_int32)
    L.wgkv_version.restype = C.c_char_p
    L.wgkv_get_meta_layout.argtypes = [C.POINTER(_CConfig), C.POINTER(_CLayout)]
    L.wgkv_query_sizes.argtypes = [C.POINTER(_CConfig), i32, i64, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    L.wgkv_init_pool.argtypes = [C.POINTER(_CConfig), vp, sz, vp, sz, vp, C.POINTER(vp)]
    L.wgkv_gate_scores.argtypes = [i32, i64, i32, i32, vp, vp, vp, vp]
    L.wgkv_gate_mlp_scores.argtypes = [i32, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp]
    L.wgkv_soft_attn_forward.argtypes = [i32, i32, pi32, i32, i32, i32, i32, vp, vp, vp, vp, f32, f32, vp, vp, vp]
    L.wgkv_soft_attn_workspace_bytes.argtypes = [i64, i32]
    L.wgkv_soft_attn_workspace_bytes.restype = sz
    L.wgkv_soft_attn_backward.argtypes = [i32, i32, pi32, i32, i32, i32, i32, vp, vp, vp, vp, f32, f32, vp, vp, vp,
                                          vp, vp, vp, vp, vp, sz, vp]
    L.wgkv_sparsity_loss.argtypes = [vp, i64, i64, vp, vp, vp, sz, vp]
    L.wgkv_prefill_admit.argtypes = [vp, i32, i32, pi32, pi32, vp, vp, vp, vp, vp, i32, f32, vp, vp, sz, vp]
    L.wgkv_decode_promote.argtypes = [vp, i32, pi32, f32, vp]
    L.wgkv_tune_decode_attention.argtypes = [vp, i32, pi32, vp, f32, vp, vp, sz, vp, C.POINTER(C.c_int32)]
    L.wgkv_prefill_admit_bounded.argtypes = [vp, i32, i32, pi32, pi32, vp, vp, vp, vp, vp, i32, f32, i32, vp, vp, sz, vp]
    L.wgkv_decode_step.argtypes = [vp, i32, i32, pi32, vp, vp, vp, f32, vp, vp]
    L.wgkv_attend.argtypes = [vp, i32, i32, pi32, pi32, vp, vp, vp, vp, f32, f32, vp, vp, sz, vp]
    L.wgkv_attend_decode_static.argtypes = [vp, i32, i32, pi32, vp, f32, vp, vp]
    L.wgkv_quest_landmark_bytes.argtypes = [C.POINTER(_CConfig), C.POINTER(sz)]
    L.wgkv_quest_update.argtypes = [vp, i32, i32, pi32, vp, sz, i32, vp]
    L.wgkv_quest_select.argtypes = [vp, i32, i32, pi32, vp, vp, sz, i32, vp, i64, vp, vp, vp]
    L.wgkv_attend_selected.argtypes = [vp, i32, i32, pi32, vp, vp, vp, i32, f32, vp, vp, sz, vp]
    L.wgkv_evict_scores.argtypes = [vp, i32, i32, pi32, vp, i32, f32, i32, vp, vp, i64, vp, sz, vp]
    L.wgkv_evict_apply.argtypes = [vp, i32, i32, pi32, vp, i64, f32, vp, vp, sz, vp]
    L.wgkv_free_seq.argtypes = [vp, i32, vp]
    L.wgkv_status.argtypes = [vp, vp, C.POINTER(i64), C.POINTER(i32)]
    L.wgkv_clear_error.argtypes = [vp, vp]
    L.wgkv_stream_read_probe.argtypes = [vp, sz, vp, vp, vp, vp]
    L.wgkv_set_profile_events.argtypes = [vp, vp, vp]
    L.wgkv_destroy.argtypes = [vp]
    L.wgkv_destroy.restype = None
    _lib = L
    return L


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _ids(xs):
    arr = (C.c_int32 * len(xs))(*[int(x) for x in xs])
    return arr


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != 0:
        raise WgkvError(rc, what)


def stream_read_probe(buf, n_bytes, sink, ev_begin=None, ev_end=None):
    """wgkv_stream_read_probe: a read-only kernel over the first n_bytes of the uint8 tensor `buf`;
    ev_begin / ev_end are raw hipEvent_t handles (ints) or None."""
    L = load_library()
    _check(L.wgkv_stream_read_probe(_ptr(buf), int(n_bytes), _ptr(sink), C.c_void_p(ev_begin) if ev_begin else None,
                                    C.c_void_p(ev_end) if ev_end else None, _stream()), "wgkv_stream_read_probe")


def gate_scores(hidden, gate_w, out=None):
    """wgkv_gate_scores: g[t][h] = sigmoid(gate_w[h] . hidden[t]) as float32 [T, Hkv]."""
    import torch
    L = load_library()
    assert hidden.is_cuda and gate_w.is_cuda and hidden.is_contiguous() and gate_w.is_contiguous()
    assert hidden.dtype == gate_w.dtype and hidden.dtype in (torch.float32, torch.bfloat16)
    T, dim = hidden.shape
    Hk = gate_w.shape[0]
    if out is None:
        out = torch.empty((T, Hk), dtype=torch.float32, device=hidden.device)
    dt = F32 if hidden.dtype == torch.float32 else BF16
    _check(L.wgkv_gate_scores(dt, T, dim, Hk, _ptr(hidden), _ptr(gate_w), _ptr(out), _stream()), "wgkv_gate_scores")
    return out


def soft_attn_forward(q, k, v, g, n_tokens, w_local, scale, eps):
    """wgkv_soft_attn_forward: training-time Write-Gated Attention of packed sequences.
    q [rows, Hq, d], k, v [rows, Hkv, d] bfloat16, g [rows, Hkv] float32, n_tokens: tokens per
    sequence.  Returns (out float32 [rows, Hq, d], lse float32 [rows, Hq])."""
    import torch
    L = load_library()
    rows, Hq, d = q.shape
    Hk = k.shape[1]
    assert k.shape == (rows, Hk, d) and v.shape == k.shape and g.shape == (rows, Hk) and sum(n_tokens) == rows
    assert q.dtype == torch.bfloat16 and k.dtype == q.dtype and v.dtype == q.dtype and g.dtype == torch.float32
    assert all(t.is_contiguous() for t in (q, k, v, g))
    out = torch.empty((rows, Hq, d), dtype=torch.float32, device=q.device)
    lse = torch.empty((rows, Hq), dtype=torch.float32, device=q.device)
    rc = L.wgkv_soft_attn_forward(BF16, len(n_tokens), _ids(n_tokens), Hq, Hk, d, int(w_local), _ptr(q), _ptr(k),
                                  _ptr(v), _ptr(g), float(scale), float(eps), _ptr(out), _ptr(lse), _stream())
    if rc:
        raise WgkvError(rc, "wgkv_soft_attn_forward")
    return out, lse


def soft_attn_backward(q, k, v, g, out, lse, dout, n_tokens, w_local, scale, eps):
    """wgkv_soft_attn_backward: (dq, dk, dv, dg) float32 for dout bfloat16 [rows, Hq, d]."""
    import torch
    L = load_library()
    rows, Hq, d = q.shape
    Hk = k.shape[1]
    assert dout.shape == q.shape and dout.dtype == torch.bfloat16 and out.dtype == torch.float32
    assert all(t.is_contiguous() for t in (q, k, v, g, out, lse, dout))
    dq = torch.empty((rows, Hq, d), dtype=torch.float32, device=q.device)
    dk = torch.empty((rows, Hk, d), dtype=torch.float32, device=q.device)
    dv = torch.empty((rows, Hk, d), dtype=torch.float32, device=q.device)
    dg = torch.empty((rows, Hk), dtype=torch.float32, device=q.device)
    nb = int(L.wgkv_soft_attn_workspace_bytes(rows, Hq))
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device=q.device)
    rc = L.wgkv_soft_attn_backward(BF16, len(n_tokens), _ids(n_tokens), Hq, Hk, d, int(w_local), _ptr(q), _ptr(k),
                                   _ptr(v), _ptr(g), float(scale), float(eps), _ptr(out), _ptr(lse), _ptr(dout),
                                   _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dg), _ptr(ws), nb, _stream())
    if rc:
        raise WgkvError(rc, "wgkv_soft_attn_backward")
    return dq, dk, dv, dg


def sparsity_loss(g, n_total=None, need_grad=True):
    """wgkv_sparsity_loss: (loss float32 [1], dg float32 like g or None) of the scores g (float32, any shape)."""
    import torch
    L = load_library()
    assert g.dtype == torch.float32 and g.is_contiguous()
    n = g.numel()
    loss = torch.empty(1, dtype=torch.float32, device=g.device)
    dg = torch.empty_like(g) if need_grad else None
    ws = torch.empty(4096, dtype=torch.uint8, device=g.device)
    rc = L.wgkv_sparsity_loss(_ptr(g), n, int(n_total if n_total is not None else n), _ptr(loss), _ptr(dg), _ptr(ws),
                              4096, _stream())
    if rc:
        raise WgkvError(rc, "wgkv_sparsity_loss")
    return loss, dg


def gate_mlp_scores(k, k_rope, w1, b1, w2, b2, eps=1e-6, out=None):
    """wgkv_gate_mlp_scores: the Write-Gate MLP on keys before / after the rotary embedding.
    k, k_rope [T, Hkv, d]; w1 [Hkv, width, 2d], w2 [Hkv, width] of the keys' dtype;
    b1 [Hkv, width], b2 [Hkv] float32.  Returns float32 [T, Hkv]."""
    import torch
    L = load_library()
    T, Hk, d = k.shape
    width = w1.shape[1]
    for x in (k, k_rope, w1, b1, w2, b2):
        assert x.is_cuda and x.is_contiguous()
    assert k_rope.shape == k.shape and w1.shape == (Hk, width, 2 * d) and w2.shape == (Hk, width)
    assert b1.shape == (Hk, width) and b2.shape == (Hk,)
    assert k.dtype in (torch.float32, torch.bfloat16) and k_rope.dtype == k.dtype
    assert w1.dtype == k.dtype and w2.dtype == k.dtype and b1.dtype == torch.float32 and b2.dtype == torch.float32
    if out is None:
        out = torch.empty((T, Hk), dtype=torch.float32, device=k.device)
    dt = F32 if k.dtype == torch.float32 else BF16
    _check(L.wgkv_gate_mlp_scores(dt, T, Hk, d, width, _ptr(k), _ptr(k_rope), _ptr(w1), _ptr(b1), _ptr(w2),
                                  _ptr(b2), eps, _ptr(out), _stream()), "wgkv_gate_mlp_scores")
    return out


class Pool:
    """Owns the torch buffers (pool, metadata, workspace) and the library handle."""

    def __init__(self, cfg: Config, max_call_seqs: int, max_call_tokens: int, device="cuda:0"):
        import torch
        self.L = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("wgkv needs a GPU: there is no CPU path")
        self.cfg = cfg
        self.device = torch.device(device)
        cc = cfg.c()
        pb, mb, wb = C.c_size_t(), C.c_size_t(), C.c_size_t()
        _check(self.L.wgkv_query_sizes(C.byref(cc), max_call_seqs, max_call_tokens, C.byref(pb),
                                       C.byref(mb), C.byref(wb)), "wgkv_query_sizes")
        self.layout = _CLayout()
        _check(self.L.wgkv_get_meta_layout(C.byref(cc), C.byref(self.layout)), "wgkv_get_meta_layout")
        self.pool_buf = torch.empty(pb.value, dtype=torch.uint8, device=self.device)
        self.meta_buf = torch.empty(mb.value, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(wb.value, dtype=torch.uint8, device=self.device)
        self.torch_dtype = torch.float32 if cfg.dtype == F32 else torch.bfloat16
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.L.wgkv_init_pool(C.byref(cc), _ptr(self.pool_buf), pb.value, _ptr(self.meta_buf),
                                         mb.value, _stream(), C.byref(h)), "wgkv_init_pool")
        self.h = h

    def __del__(self):
        if getattr(self, "h", None):
            self.L.wgkv_destroy(self.h)
            self.h = None

    # ---- the path ----
    def prefill_admit(self, layer, seq_ids, n_tokens, k, v, g=None, hidden=None, gate_w=None,
                      tau=0.5, admit_mask_out=None, max_admitted_per_head=None):
        """wgkv_prefill_admit, or wgkv_prefill_admit_bounded when max_admitted_per_head is given."""
        hd = 0 if hidden is None else hidden.shape[-1]
        if max_admitted_per_head is None:
            _check(self.L.wgkv_prefill_admit(self.h, layer, len(seq_ids), _ids(seq_ids), _ids(n_tokens),
                                             _ptr(k), _ptr(v), _ptr(g), _ptr(hidden), _ptr(gate_w), hd,
                                             tau, _ptr(admit_mask_out), _ptr(self.workspace),
                                             self.workspace.numel(), _stream()), "wgkv_prefill_admit")
        else:
            _check(self.L.wgkv_prefill_admit_bounded(self.h, layer, len(seq_ids), _ids(seq_ids), _ids(n_tokens),
                                                     _ptr(k), _ptr(v), _ptr(g), _ptr(hidden), _ptr(gate_w), hd,
                                                     tau, int(max_admitted_per_head), _ptr(admit_mask_out),
                                                     _ptr(self.workspace), self.workspace.numel(), _stream()),
                   "wgkv_prefill_admit_bounded")

    def decode_step(self, layer, seq_ids, k_new, v_new, g_new, tau=0.5, promoted_out=None):
        _check(self.L.wgkv_decode_step(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(k_new),
                                       _ptr(v_new), _ptr(g_new), tau, _ptr(promoted_out), _stream()),
               "wgkv_decode_step")

    def decode_promote(self, seq_ids, tau=0.5):
        """wgkv_decode_promote: victim test, page hand-out and row move of every layer, ahead of the layers' steps."""
        _check(self.L.wgkv_decode_promote(self.h, len(seq_ids), _ids(seq_ids), tau, _stream()), "wgkv_decode_promote")

    def attend(self, layer, seq_ids, q, out, scale, n_q=None, k_chunk=None, v_chunk=None,
               g_chunk=None, tau=0.5):
        if n_q is None:
            n_q = [1] * len(seq_ids)
        _check(self.L.wgkv_attend(self.h, layer, len(seq_ids), _ids(seq_ids), _ids(n_q), _ptr(q),
                                  _ptr(k_chunk), _ptr(v_chunk), _ptr(g_chunk), tau, scale, _ptr(out),
                                  _ptr(self.workspace), self.workspace.numel(), _stream()), "wgkv_attend")
        return out

    def tune_decode_attention(self, seq_ids, q, out, scale):
        """wgkv_tune_decode_attention: picks the odd/even XCD correction of the tile split on this machine; returns it."""
        kept = C.c_int32(-1)
        _check(self.L.wgkv_tune_decode_attention(self.h, len(seq_ids), _ids(seq_ids), _ptr(q), scale, _ptr(out),
                                                 _ptr(self.workspace), self.workspace.numel(), _stream(),
                                                 C.byref(kept)), "wgkv_tune_decode_attention")
        return kept.value

    def attend_decode_static(self, layer, seq_ids, q, out, scale):
        """wgkv_attend_decode_static: decode attention without a workspace argument."""
        _check(self.L.wgkv_attend_decode_static(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(q), scale,
                                                _ptr(out), _stream()), "wgkv_attend_decode_static")
        return out

    def quest_landmarks(self):
        """A zero-filled landmark buffer of the size the library asks for (uint8 tensor)."""
        import torch
        n = C.c_size_t(0)
        cc = self.cfg.c()
        _check(self.L.wgkv_quest_landmark_bytes(C.byref(cc), C.byref(n)), "wgkv_quest_landmark_bytes")
        return torch.zeros(n.value, dtype=torch.uint8, device=self.device)

    def quest_update(self, layer, seq_ids, landmarks, reset=False):
        _check(self.L.wgkv_quest_update(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(landmarks), landmarks.numel(),
                                        1 if reset else 0, _stream()), "wgkv_quest_update")

    def quest_select(self, layer, seq_ids, q, landmarks, budget_pages, score_stride, scores=None):
        """Returns (page_scores [n_units, score_stride], sel_pages int32 [n_units, budget_pages], sel_count [n_units]).
        scores: the caller's own contiguous float32 buffer of n_units * score_stride elements, else a new one."""
        import torch
        n_units = len(seq_ids) * self.cfg.n_kv_heads
        if scores is None:
            scores = torch.zeros((n_units, score_stride), dtype=torch.float32, device=self.device)
        assert scores.is_cuda and scores.is_contiguous() and scores.dtype == torch.float32
        assert scores.numel() == n_units * score_stride
        sel = torch.full((n_units, budget_pages), -1, dtype=torch.int32, device=self.device)
        cnt = torch.zeros((n_units,), dtype=torch.int32, device=self.device)
        _check(self.L.wgkv_quest_select(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(q), _ptr(landmarks),
                                        landmarks.numel(), budget_pages, _ptr(scores), score_stride, _ptr(sel),
                                        _ptr(cnt), _stream()), "wgkv_quest_select")
        return scores, sel, cnt

    def attend_selected(self, layer, seq_ids, q, sel_pages, sel_count, out, scale):
        _check(self.L.wgkv_attend_selected(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(q), _ptr(sel_pages),
                                           _ptr(sel_count), sel_pages.shape[1], scale, _ptr(out), _ptr(self.workspace),
                                           self.workspace.numel(), _stream()), "wgkv_attend_selected")
        return out

    def evict_scores(self, layer, seq_ids, q_obs, scale, stride, pool_w=5):
        """wgkv_evict_scores: q_obs [len(seq_ids), n_obs, n_q_heads, d]; returns (raw, pooled), float32
        [len(seq_ids) * n_kv_heads, stride], rows valid up to each head's global length."""
        import torch
        assert q_obs.is_cuda and q_obs.is_contiguous() and q_obs.dim() == 4 and q_obs.shape[0] == len(seq_ids)
        n_units = len(seq_ids) * self.cfg.n_kv_heads
        raw = torch.zeros((n_units, stride), dtype=torch.float32, device=self.device)
        out = torch.zeros((n_units, stride), dtype=torch.float32, device=self.device)
        _check(self.L.wgkv_evict_scores(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(q_obs), q_obs.shape[1],
                                        scale, pool_w, _ptr(raw), _ptr(out), stride, _ptr(self.workspace),
                                        self.workspace.numel(), _stream()), "wgkv_evict_scores")
        return raw, out

    def evict_apply(self, layer, seq_ids, scores, frac, n_evicted_out=None):
        """wgkv_evict_apply: scores float32 [len(seq_ids) * n_kv_heads, stride] on the device."""
        import torch
        assert scores.is_cuda and scores.is_contiguous() and scores.dtype == torch.float32 and scores.dim() == 2
        assert scores.shape[0] == len(seq_ids) * self.cfg.n_kv_heads
        _check(self.L.wgkv_evict_apply(self.h, layer, len(seq_ids), _ids(seq_ids), _ptr(scores), scores.shape[1],
                                       frac, _ptr(n_evicted_out), _ptr(self.workspace), self.workspace.numel(),
                                       _stream()), "wgkv_evict_apply")

    def free_seq(self, seq_id):
        _check(self.L.wgkv_free_seq(self.h, seq_id, _stream()), "wgkv_free_seq")

    def status(self):
        free, flag = C.c_int64(), C.c_int32()
        rc = self.L.wgkv_status(self.h, _stream(), C.byref(free), C.byref(flag))
        if rc not in (0, -5):
            raise WgkvError(rc, "wgkv_status")
        return free.value, flag.value

    def clear_error(self):
        _check(self.L.wgkv_clear_error(self.h, _stream()), "wgkv_clear_error")

    def set_profile_events(self, ev_begin, ev_end):
        """ev_begin/ev_end: raw hipEvent_t handles (ints) or None."""
        _check(self.L.wgkv_set_profile_events(self.h, C.c_void_p(ev_begin) if ev_begin else None,
                                              C.c_void_p(ev_end) if ev_end else None),
               "wgkv_set_profile_events")

    # ---- views of the documented metadata layout (inspection / snapshots) ----
    def _view(self, off, count, dtype):
        import torch
        es = 4
        return self.meta_buf[off: off + count * es].view(dtype)

    def meta(self):
        import torch
        c, lay = self.cfg, self.layout
        S, Lr, H, W = c.max_seqs, c.n_layers, c.n_kv_heads, c.w_local
        nlp, mgp = lay.n_local_pages, c.max_global_pages_per_head
        i32, f32 = torch.int32, torch.float32
        return {
            "seq_len": self._view(lay.seq_len, S * Lr, i32).view(S, Lr),
            "global_len": self._view(lay.global_len, S * Lr * H, i32).view(S, Lr, H),
            "local_pt": self._view(lay.local_pt, S * Lr * H * nlp, i32).view(S, Lr, H, nlp),
            "global_pt": self._view(lay.global_pt, S * Lr * H * mgp, i32).view(S, Lr, H, mgp),
            "ring_g": self._view(lay.ring_g, S * Lr * H * W, f32).view(S, Lr, H, W),
            "free_stack": self._view(lay.free_stack, c.n_pages, i32),
            "free_top": self._view(lay.free_top, 1, i32),
            "err_flag": self._view(lay.err_flag, 1, i32),
        }

    def pool_pages(self):
        """The pool as [n_pages, 2 (K,V), P, head_dim] in the pool dtype."""
        c = self.cfg
        return self.pool_buf.view(self.torch_dtype).view(c.n_pages, 2, c.page_size, c.head_dim)
