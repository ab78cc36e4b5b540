"""ctypes binding of libspin.so.  Same names as the C ABI (include/spin.h), minus the prefix.

Marshalling only: numpy int32 arrays for host tables, torch tensors for device memory
(`data_ptr()`), the current torch stream for launches.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

OK, EINVAL, ETABLE, ENOSPC, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4, -5
DECOMP_NONE, DECOMP_Q_SPLIT, DECOMP_KV_SPLIT, DECOMP_KV_SEARCH = 0, 1, 2, 3
ACCEPT_GREEDY, ACCEPT_REJECTION = 0, 1
DTYPE_BF16 = 1
DTYPE_F16 = 2

SUBREQ_DTYPE = np.dtype([("parent", "<i4"), ("q_begin", "<i4"), ("q_len", "<i4"),
                         ("kv_begin", "<i4"), ("kv_len", "<i4")])

_i32p = C.POINTER(C.c_int32)
_i64p = C.POINTER(C.c_int64)


class ReqTable(C.Structure):
    _fields_ = [("n_req", C.c_int32), ("prefix_len", _i32p), ("draft_len", _i32p),
                ("q_offset", _i32p), ("pt_offset", _i32p), ("page_table", _i32p)]


class KvDesc(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("n_pages", C.c_int32),
                ("page_size", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_stride", C.c_int64), ("head_stride", C.c_int64), ("token_stride", C.c_int64),
                ("dtype", C.c_int32)]


class SubReq(C.Structure):
    _fields_ = [("parent", C.c_int32), ("q_begin", C.c_int32), ("q_len", C.c_int32),
                ("kv_begin", C.c_int32), ("kv_len", C.c_int32)]


class WorkPiece(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("parent", "q_begin", "q_len", "kv_begin", "kv_len", "kv_head",
                                          "tile_class", "wave", "flags")]


PIECE_CARRY_IN, PIECE_CARRY_OUT, PIECE_DIRECT, PIECE_QUEUED = 1, 2, 4, 8


class DecompParams(C.Structure):
    _fields_ = [("policy", C.c_int32), ("q_width", C.c_int32), ("kv_len", C.c_int32),
                ("max_subreq", C.c_int32), ("l_min", C.c_int32), ("l_max", C.c_int32),
                ("l_step", C.c_int32)]


class SpinError(RuntimeError):
    def __init__(self, code: int, text: str = ""):
        self.code = code
        super().__init__(f"libspin error {code}: {text}")


EXPORTS = ["spin_create", "spin_reserve", "spin_required", "spin_destroy", "spin_strerror",
           "spin_last_error", "spin_set_waves", "spin_decompose", "spin_kv_padding",
           "spin_check_tiling", "spin_schedule", "spin_verify_attn", "spin_verify_attn_tree", "spin_append_kv", "spin_accept", "spin_accept_noalloc", "spin_accept_tree",
           "spin_set_plan_reuse", "spin_profile_begin", "spin_profile_every", "spin_profile_end"]

_lib = None


def lib_path() -> str:
    # SPIN_LIB names another build of the library (for comparing two builds in one session)
    return os.environ.get("SPIN_LIB") or os.path.join(HERE, "libspin.so")


def load_library():
    """Load libspin.so (built in-tree by paper_2503_15921_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2503_15921_amd.build`")
    lib = C.CDLL(path)
    sp = C.POINTER(SubReq)
    tp = C.POINTER(ReqTable)
    lib.spin_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
    lib.spin_reserve.argtypes = [C.c_void_p] + [C.c_int64] * 5
    lib.spin_required.argtypes = [C.c_void_p] + [_i64p] * 5
    lib.spin_destroy.argtypes = [C.c_void_p]
    lib.spin_destroy.restype = None
    lib.spin_strerror.argtypes = [C.c_int]
    lib.spin_strerror.restype = C.c_char_p
    lib.spin_last_error.argtypes = [C.c_void_p, C.c_char_p, C.c_size_t]
    lib.spin_set_waves.argtypes = [C.c_void_p, C.c_int32]
    lib.spin_decompose.argtypes = [tp, C.POINTER(DecompParams), sp, C.c_int32, _i32p, _i32p]
    lib.spin_kv_padding.argtypes = [tp, C.c_int32, _i64p, _i64p]
    lib.spin_check_tiling.argtypes = [tp, sp, C.c_int32]
    lib.spin_schedule.argtypes = [tp, sp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                  C.POINTER(WorkPiece), C.c_int32, _i32p]
    lib.spin_verify_attn.argtypes = [C.c_void_p, C.POINTER(KvDesc), tp, sp, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
    lib.spin_verify_attn_tree.argtypes = [C.c_void_p, C.POINTER(KvDesc), tp, sp, C.c_int32, C.POINTER(C.c_uint64),
                                          C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
    lib.spin_append_kv.argtypes = [C.c_void_p, C.POINTER(KvDesc), tp, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.spin_accept.argtypes = [C.c_void_p, C.c_int32, C.c_int32, _i32p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p]
    lib.spin_accept_noalloc.argtypes = [C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 4 + [C.c_int32] + [C.c_void_p] * 5
    lib.spin_accept_tree.argtypes = [C.c_void_p, C.c_int32, C.c_int32, _i32p, _i32p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.spin_set_plan_reuse.argtypes = [C.c_void_p, C.c_int32]
    lib.spin_profile_begin.argtypes = [C.c_void_p, C.c_int32]
    lib.spin_profile_every.argtypes = [C.c_void_p, C.c_int32]
    lib.spin_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_double), _i32p]
    for name in EXPORTS:
        if name not in ("spin_destroy", "spin_strerror"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_i32p)


class _Table:
    """Keeps the numpy arrays alive while the C struct points at them."""

    def __init__(self, prefix_len, draft_len, q_offset=None, pt_offset=None, page_table=None):
        self.prefix_len = _i32(prefix_len)
        self.draft_len = _i32(draft_len)
        n = self.prefix_len.shape[0]
        if q_offset is None:
            q_offset = np.concatenate([[0], np.cumsum(self.draft_len, dtype=np.int64)])
        self.q_offset = _i32(q_offset)
        self.pt_offset = None if pt_offset is None else _i32(pt_offset)
        self.page_table = None if page_table is None else _i32(page_table)
        self.struct = ReqTable(n, _ptr(self.prefix_len), _ptr(self.draft_len), _ptr(self.q_offset),
                               _ptr(self.pt_offset), _ptr(self.page_table))


def _subs_arg(subs):
    if subs is None:
        return None, 0, None
    arr = np.ascontiguousarray(np.asarray(subs, dtype=np.int32).reshape(-1, 5))
    return arr.ctypes.data_as(C.POINTER(SubReq)), arr.shape[0], arr


def _check(rc: int, ctx=None):
    if rc == 0:
        return
    lib = load_library()
    text = lib.spin_strerror(rc).decode()
    if ctx is not None:
        buf = C.create_string_buffer(512)
        lib.spin_last_error(ctx, buf, 512)
        if buf.value:
            text += ": " + buf.value.decode()
    raise SpinError(rc, text)


# ----------------------------------------------------------------------------- host-only calls
def decompose(prefix_len, draft_len, policy: int, q_width: int = 0, kv_len: int = 0, max_subreq: int = 0,
              l_min: int = 0, l_max: int = 0, l_step: int = 1, cap: Optional[int] = None):
    """spin_decompose.  Returns (int32 array [n,5] of (parent,q_begin,q_len,kv_begin,kv_len), chosen L)."""
    lib = load_library()
    t = _Table(prefix_len, draft_len)
    params = DecompParams(policy, q_width, kv_len, max_subreq, l_min, l_max, l_step)
    n = C.c_int32(0)
    L = C.c_int32(0)
    if cap is None:
        rc = lib.spin_decompose(C.byref(t.struct), C.byref(params), None, 0, C.byref(n), C.byref(L))
        if rc not in (OK, ENOSPC) or (rc == ENOSPC and n.value == 0):
            _check(rc)
        cap = n.value
    out = np.zeros((max(cap, 1), 5), dtype=np.int32)
    rc = lib.spin_decompose(C.byref(t.struct), C.byref(params), out.ctypes.data_as(C.POINTER(SubReq)), cap,
                            C.byref(n), C.byref(L))
    _check(rc)
    return out[: n.value].copy(), L.value


def kv_padding(prefix_len, draft_len, kv_len: int):
    lib = load_library()
    t = _Table(prefix_len, draft_len)
    rows, pad = C.c_int64(0), C.c_int64(0)
    _check(lib.spin_kv_padding(C.byref(t.struct), kv_len, C.byref(rows), C.byref(pad)))
    return rows.value, pad.value


def check_tiling(prefix_len, draft_len, subs) -> int:
    """spin_check_tiling: returns the error code (0 = exact tiling) instead of raising."""
    lib = load_library()
    t = _Table(prefix_len, draft_len)
    p, n, keep = _subs_arg(subs)
    return lib.spin_check_tiling(C.byref(t.struct), p, n)


def schedule(prefix_len, draft_len, subs, page_size: int, group: int, n_kv_heads: int, n_waves: int) -> np.ndarray:
    """spin_schedule: the pieces the attention kernel would stream, as an int32 [n,9] array of
    (parent, q_begin, q_len, kv_begin, kv_len, kv_head, tile_class, wave, flags)."""
    lib = load_library()
    t = _Table(prefix_len, draft_len)
    p, n, keep = _subs_arg(subs)
    cnt = C.c_int32(0)
    rc = lib.spin_schedule(C.byref(t.struct), p, n, page_size, group, n_kv_heads, n_waves, None, 0, C.byref(cnt))
    if rc not in (OK, ENOSPC):
        _check(rc)
    out = np.zeros((max(cnt.value, 1), 9), dtype=np.int32)
    _check(lib.spin_schedule(C.byref(t.struct), p, n, page_size, group, n_kv_heads, n_waves,
                             out.ctypes.data_as(C.POINTER(WorkPiece)), cnt.value, C.byref(cnt)))
    return out[: cnt.value].copy()


def accept_noalloc(mode: int, q_offset_dev, draft_tokens, target_logits, draft_logits, u_accept, u_sample,
                   n_accepted, next_token, n_rows: Optional[int] = None, stream=None) -> None:
    """spin_accept_noalloc: spin_accept without a context and without any allocation.  q_offset_dev: torch
    int32 device tensor [n_req+1]; the other tensors as in SpinContext.accept."""
    import torch
    lib = load_library()
    n_req = q_offset_dev.shape[0] - 1
    if n_rows is None:
        n_rows = draft_tokens.shape[0]
    dev = target_logits.device.index or 0
    st = C.c_void_p(torch._C._cuda_getCurrentRawStream(dev) if stream is None else stream.cuda_stream)

    def ptr(t):
        return C.c_void_p(None if t is None else t.data_ptr())
    with torch.cuda.device(dev):
        _check(lib.spin_accept_noalloc(mode, n_req, n_rows, ptr(q_offset_dev), ptr(draft_tokens), ptr(target_logits),
                                       ptr(draft_logits), target_logits.shape[-1], ptr(u_accept), ptr(u_sample),
                                       ptr(n_accepted), ptr(next_token), st))


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    if t.dtype == torch.float16:
        return DTYPE_F16
    raise TypeError(f"K/V must be torch.bfloat16 or torch.float16, not {t.dtype}")


# ----------------------------------------------------------------------------- GPU context
class SpinContext:
    """Owns a spin_ctx.  `auto_reserve` lets the binding grow the workspace when a call reports
    SPIN_ENOSPC (the library itself never allocates on the hot path)."""

    def __init__(self, device: int = 0, auto_reserve: bool = True):
        self._lib = load_library()
        h = C.c_void_p()
        _check(self._lib.spin_create(C.byref(h), device))
        self._h = h
        self._device = device
        self.auto_reserve = auto_reserve

    def close(self):
        if getattr(self, "_h", None):
            self._lib.spin_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reserve(self, max_req, max_rows, max_pages, max_items, max_part_slots):
        _check(self._lib.spin_reserve(self._h, max_req, max_rows, max_pages, max_items, max_part_slots), self._h)

    def required(self):
        v = [C.c_int64(0) for _ in range(5)]
        _check(self._lib.spin_required(self._h, *[C.byref(x) for x in v]), self._h)
        return tuple(x.value for x in v)

    def set_waves(self, n_waves: int):
        _check(self._lib.spin_set_waves(self._h, n_waves), self._h)

    def accept_tree(self, mode: int, draft_len, parents, draft_tokens, target_logits, draft_logits, u_accept, u_sample,
                    n_accepted, path, next_token, stream=None):
        """spin_accept_tree.  draft_len, parents: host int32; the rest torch device tensors (draft_logits and
        the uniforms may be None in greedy mode)."""
        dl = _i32(draft_len)
        par = _i32(parents)
        vocab = target_logits.shape[-1]
        st = self._stream(stream)

        def ptr(t):
            return C.c_void_p(None if t is None else t.data_ptr())
        self._retry(lambda: self._lib.spin_accept_tree(
            self._h, mode, dl.shape[0], _ptr(dl), _ptr(par), ptr(draft_tokens), ptr(target_logits), ptr(draft_logits),
            vocab, ptr(u_accept), ptr(u_sample), ptr(n_accepted), ptr(path), ptr(next_token), st))

    def set_plan_reuse(self, enable: bool):
        """Whether a call with the same tables as the previous one launches from the tables already staged."""
        _check(self._lib.spin_set_plan_reuse(self._h, 1 if enable else 0), self._h)

    def profile_begin(self, max_calls: int, every: int = 1):
        """Time up to max_calls calls of each kind, every `every`-th call seen."""
        _check(self._lib.spin_profile_every(self._h, every), self._h)
        _check(self._lib.spin_profile_begin(self._h, max_calls), self._h)

    def profile_end(self):
        """Returns ({'attn','join','accept_stats','accept_draw'} -> summed ms, (attn calls, accept calls))."""
        ms = (C.c_double * 4)()
        calls = (C.c_int32 * 2)()
        _check(self._lib.spin_profile_end(self._h, ms, calls), self._h)
        return dict(attn=ms[0], join=ms[1], accept_stats=ms[2], accept_draw=ms[3]), (calls[0], calls[1])

    def _retry(self, call):
        rc = call()
        if rc == ENOSPC and self.auto_reserve:
            need = self.required()
            self.reserve(*[int(x * 1.25) + 16 for x in need])
            rc = call()
        _check(rc, self._h)

    def _stream(self, stream):
        import torch
        if stream is None:
            # the raw handle of torch's current stream on the context's device (torch.cuda.current_stream()
            # builds a Stream object and costs several microseconds per call)
            return C.c_void_p(torch._C._cuda_getCurrentRawStream(self._device))
        return C.c_void_p(stream.cuda_stream)

    def make_table(self, prefix_len, draft_len, q_offset, pt_offset, page_table) -> _Table:
        return _Table(prefix_len, draft_len, q_offset, pt_offset, page_table)

    def verify_attn(self, table: _Table, k_pool, v_pool, q, out, n_q_heads: int, subs=None,
                    softmax_scale: float = 0.0, page_size: Optional[int] = None, stream=None,
                    strides=None, tree_mask=None):
        """spin_verify_attn, or spin_verify_attn_tree when tree_mask (host uint64 [R]) is given.  k_pool/v_pool: torch bf16 or fp16 [n_pages][n_kv_heads][page_size][head_dim]
        (or any layout with `strides` = (page, head, token) in elements and page_size given);
        q/out: torch tensors of the same type, [R][n_q_heads][head_dim]."""
        assert q.dtype == k_pool.dtype == v_pool.dtype == out.dtype
        if strides is None:
            n_pages, n_kv, psz, d = k_pool.shape
            ps, hs, ts, ds = k_pool.stride()
            assert ds == 1 and tuple(v_pool.stride()) == tuple(k_pool.stride())
        else:
            n_pages, n_kv, psz, d = k_pool.shape
            ps, hs, ts = strides
        if page_size is not None:
            psz = page_size
        desc = KvDesc(k_pool.data_ptr(), v_pool.data_ptr(), n_pages, psz, n_kv, d, ps, hs, ts, _dtype_code(k_pool))
        sp, ns, keep = _subs_arg(subs)
        st = self._stream(stream)
        if tree_mask is not None:
            tm = np.ascontiguousarray(tree_mask, dtype=np.uint64)
            assert tm.shape == (q.shape[0],)
            self._retry(lambda: self._lib.spin_verify_attn_tree(
                self._h, C.byref(desc), C.byref(table.struct), sp, ns, tm.ctypes.data_as(C.POINTER(C.c_uint64)),
                C.c_void_p(q.data_ptr()), C.c_void_p(out.data_ptr()), n_q_heads, softmax_scale, st))
            return
        self._retry(lambda: self._lib.spin_verify_attn(self._h, C.byref(desc), C.byref(table.struct), sp, ns,
                                                       C.c_void_p(q.data_ptr()), C.c_void_p(out.data_ptr()),
                                                       n_q_heads, softmax_scale, st))

    def append_kv(self, table: _Table, k_pool, v_pool, k_new, v_new, stream=None):
        """spin_append_kv: scatter the draft tokens' K/V rows ([R][n_kv_heads][head_dim], the pools' type) into the pools."""
        assert k_new.dtype == v_new.dtype == k_pool.dtype == v_pool.dtype
        n_pages, n_kv, psz, d = k_pool.shape
        ps, hs, ts, ds = k_pool.stride()
        assert ds == 1 and tuple(v_pool.stride()) == tuple(k_pool.stride())
        desc = KvDesc(k_pool.data_ptr(), v_pool.data_ptr(), n_pages, psz, n_kv, d, ps, hs, ts, _dtype_code(k_pool))
        st = self._stream(stream)
        self._retry(lambda: self._lib.spin_append_kv(self._h, C.byref(desc), C.byref(table.struct),
                                                     C.c_void_p(k_new.data_ptr()), C.c_void_p(v_new.data_ptr()), st))

    def accept(self, mode: int, draft_len, draft_tokens, target_logits, draft_logits, u_accept, u_sample,
               n_accepted, next_token, stream=None):
        """spin_accept.  draft_len: host int32; everything else torch device tensors."""
        dl = _i32(draft_len)
        vocab = target_logits.shape[-1]
        st = self._stream(stream)

        def ptr(t):
            return C.c_void_p(None if t is None else t.data_ptr())
        self._retry(lambda: self._lib.spin_accept(self._h, mode, dl.shape[0], _ptr(dl), ptr(draft_tokens),
                                                  ptr(target_logits), ptr(draft_logits), vocab, ptr(u_accept),
                                                  ptr(u_sample), ptr(n_accepted), ptr(next_token), st))
