"""ctypes binding of libbc.so (see include/bc.h).

Two layers, both argument marshalling only:
  * module-level functions named exactly like the C entry points, taking ctypes
    structures and raw device addresses;
  * `Runtime`, which owns the torch tensors (slabs, tables, workspace) a cache needs
    and passes their addresses and torch's current stream to those functions.
Every step of the path runs in the library's kernels; there is no fallback: loading
fails loudly when libbc.so is missing.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbc.so")
DIAG_LIB_PATH = os.path.join(_HERE, "libbc_diag.so")     # measurement aids (include/bc_diag.h)

BC_OK = 0
BC_ERR_ARG, BC_ERR_SHAPE, BC_ERR_CAPACITY, BC_ERR_STATE, BC_ERR_WORKSPACE, BC_ERR_HIP = -1, -2, -3, -4, -5, -6
BC_F32, BC_BF16 = 0, 1
BC_ERRBIT_STATE, BC_ERRBIT_CAPACITY = 1, 2
BC_ROW_TOKEN, BC_ROW_BEACON = 0, 1
# bits of bc_cache.plan
BC_PLAN_PLAIN_ALU, BC_PLAN_NEED_MATRIX_KERNEL, BC_PLAN_IGNORE_ORDER, BC_PLAN_CACHEABLE_LOADS = 1, 2, 4, 8
BC_PLAN_ONE_WORKGROUP_PER_PAIR, BC_PLAN_IGNORE_PROMISE, BC_PLAN_NO_SMALL_WORKGROUPS = 16, 32, 64
BC_PLAN_GENERAL_LOOP = 128

EXPORTS = [
    "bc_status_str", "bc_version", "bc_cache_init", "bc_cache_admit", "bc_append_kv",
    "bc_decode_workspace_bytes", "bc_workspace_init", "bc_decode_plan_describe", "bc_decode_attn",
    "bc_compress_evict", "bc_decode_step", "bc_decode_step_noalloc", "bc_beacon_step", "bc_decode_step_budget", "bc_set_ratio",
    "bc_sort_by_length",
    "bc_prefill_attn", "bc_prefill_workspace_bytes", "bc_prefill_attn_ws",
    "bc_prefill_bwd_workspace_bytes", "bc_prefill_attn_bwd",
    "bc_topk_kl_loss", "bc_topk_kl_loss_bwd", "bc_tables_to_host",
]
DIAG_EXPORTS = ["bc_diag_stream_read"]


class bc_shape(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("kv_dtype", C.c_int32), ("scale", C.c_float)]


class bc_cache(C.Structure):
    _fields_ = [("k_slab", C.c_void_p), ("v_slab", C.c_void_p), ("base", C.c_void_p),
                ("cap", C.c_void_p), ("P", C.c_void_p), ("c", C.c_void_p),
                ("nb", C.c_void_p), ("w", C.c_void_p), ("err", C.c_void_p),
                ("max_cap", C.c_int32), ("order", C.c_void_p),
                ("uniform_P", C.c_int32), ("uniform_cap", C.c_int32),
                ("rows_per_workgroup", C.c_int32), ("plan", C.c_int32)]


class BcError(RuntimeError):
    pass


_lib = None


def load():
    """Load libbc.so and declare the signatures; raises if the library or a symbol is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise BcError("libbc.so not built: run `python __graft_entry__.py` (hipcc, gfx950) first")
    lib = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        if not hasattr(lib, name):
            raise BcError("libbc.so lacks symbol %s" % name)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    sp, cp = C.POINTER(bc_shape), C.POINTER(bc_cache)
    lib.bc_status_str.restype = C.c_char_p
    lib.bc_status_str.argtypes = [i32]
    lib.bc_version.restype = i32
    lib.bc_cache_init.restype = i32
    lib.bc_cache_init.argtypes = [sp, cp, vp, vp, vp, i64, vp]
    lib.bc_cache_admit.restype = i32
    lib.bc_cache_admit.argtypes = [sp, cp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.bc_sort_by_length.restype = i32
    lib.bc_sort_by_length.argtypes = [sp, cp, vp, vp, vp]
    lib.bc_append_kv.restype = i32
    lib.bc_append_kv.argtypes = [sp, cp, vp, vp, vp, i32, vp]
    lib.bc_decode_workspace_bytes.restype = sz
    lib.bc_decode_workspace_bytes.argtypes = [sp, i32]
    lib.bc_workspace_init.restype = i32
    lib.bc_workspace_init.argtypes = [vp, sz, vp]
    lib.bc_decode_plan_describe.restype = i32
    lib.bc_decode_plan_describe.argtypes = [sp, cp, C.c_char_p, sz]
    lib.bc_decode_attn.restype = i32
    lib.bc_decode_attn.argtypes = [sp, cp, vp, vp, vp, vp, sz, vp]
    lib.bc_compress_evict.restype = i32
    lib.bc_compress_evict.argtypes = [sp, cp, vp, vp, vp, i32, vp]
    lib.bc_decode_step.restype = i32
    lib.bc_decode_step.argtypes = [sp, cp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.bc_decode_step_noalloc.restype = i32
    lib.bc_decode_step_noalloc.argtypes = [sp, cp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.bc_beacon_step.restype = i32
    lib.bc_beacon_step.argtypes = [sp, cp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.bc_decode_step_budget.restype = i32
    lib.bc_decode_step_budget.argtypes = [sp, cp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.bc_set_ratio.restype = i32
    lib.bc_set_ratio.argtypes = [sp, cp, vp, vp, vp]
    lib.bc_prefill_attn.restype = i32
    lib.bc_prefill_attn.argtypes = [sp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.bc_prefill_workspace_bytes.restype = C.c_size_t
    lib.bc_prefill_workspace_bytes.argtypes = [sp, C.c_int64]
    lib.bc_prefill_attn_ws.restype = i32
    lib.bc_prefill_attn_ws.argtypes = [sp, vp, vp, vp, vp, vp, vp, i32, C.c_int64, vp, vp, vp, C.c_size_t, vp]
    lib.bc_prefill_bwd_workspace_bytes.restype = sz
    lib.bc_prefill_bwd_workspace_bytes.argtypes = [sp, i64]
    lib.bc_prefill_attn_bwd.restype = i32
    lib.bc_prefill_attn_bwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp, vp, sz, vp]
    lib.bc_topk_kl_loss.restype = i32
    lib.bc_topk_kl_loss.argtypes = [i64, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.bc_topk_kl_loss_bwd.restype = i32
    lib.bc_topk_kl_loss_bwd.argtypes = [i64, i32, i32, vp, i32, vp, vp, vp, C.c_float, vp, vp]
    lib.bc_tables_to_host.restype = i32
    lib.bc_tables_to_host.argtypes = [sp, cp, vp, vp, vp, vp]
    _lib = lib
    return lib


_diag = None


def load_diag():
    """Load libbc_diag.so (measurement aids, see include/bc_diag.h); raises if it is missing."""
    global _diag
    if _diag is not None:
        return _diag
    if not os.path.exists(DIAG_LIB_PATH):
        raise BcError("libbc_diag.so not built: run `python __graft_entry__.py` first")
    lib = C.CDLL(DIAG_LIB_PATH)
    for name in DIAG_EXPORTS:
        if not hasattr(lib, name):
            raise BcError("libbc_diag.so lacks symbol %s" % name)
    lib.bc_diag_stream_read.restype = C.c_int32
    lib.bc_diag_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    _diag = lib
    return lib


def _check(st):
    if st != BC_OK:
        raise BcError("bc status %d: %s" % (st, load().bc_status_str(st).decode()))


def bc_status_str(st):
    return load().bc_status_str(st).decode()


def bc_version():
    return load().bc_version()


def bc_cache_init(shape, cache, k_prompt, v_prompt, prompt_offsets, total_rows, stream):
    return load().bc_cache_init(C.byref(shape), C.byref(cache), k_prompt, v_prompt, prompt_offsets,
                                total_rows, stream)


def bc_cache_admit(shape, cache, k_prompt, v_prompt, prompt_offsets, total_rows, new_c, admit, live, stream):
    return load().bc_cache_admit(C.byref(shape), C.byref(cache), k_prompt, v_prompt, prompt_offsets,
                                 total_rows, new_c, admit, live, stream)


def bc_append_kv(shape, cache, k, v, active, kind, stream):
    return load().bc_append_kv(C.byref(shape), C.byref(cache), k, v, active, kind, stream)


def bc_decode_workspace_bytes(shape, max_cap):
    return load().bc_decode_workspace_bytes(C.byref(shape), max_cap)


def bc_workspace_init(ws, nbytes, stream):
    return load().bc_workspace_init(ws, nbytes, stream)


def bc_decode_plan_describe(shape, cache):
    """-> (status, text): the kernel, grid and chunking the decode calls use for this shape and cache."""
    buf = C.create_string_buffer(512)
    st = load().bc_decode_plan_describe(C.byref(shape), C.byref(cache), buf, len(buf))
    return st, buf.value.decode()


def bc_decode_attn(shape, cache, q, out, active, ws, ws_bytes, stream):
    return load().bc_decode_attn(C.byref(shape), C.byref(cache), q, out, active, ws, ws_bytes, stream)


def bc_compress_evict(shape, cache, beacon_k, beacon_v, active, require_full_window, stream):
    return load().bc_compress_evict(C.byref(shape), C.byref(cache), beacon_k, beacon_v, active,
                                    require_full_window, stream)


def bc_decode_step(shape, cache, k, v, q, out, beacon_k, beacon_v, active, ws, ws_bytes, stream):
    return load().bc_decode_step(C.byref(shape), C.byref(cache), k, v, q, out, beacon_k, beacon_v,
                                 active, ws, ws_bytes, stream)


def bc_decode_step_noalloc(shape, cache, k, v, q, out, beacon_k, beacon_v, active, stream):
    return load().bc_decode_step_noalloc(C.byref(shape), C.byref(cache), k, v, q, out, beacon_k, beacon_v,
                                         active, stream)


def bc_beacon_step(shape, cache, k, v, q, out, active, ws, ws_bytes, stream):
    return load().bc_beacon_step(C.byref(shape), C.byref(cache), k, v, q, out, active, ws, ws_bytes, stream)


def bc_decode_step_budget(shape, cache, k, v, q, out, beacon_k, beacon_v, budget, live, ws, ws_bytes,
                          stream):
    return load().bc_decode_step_budget(C.byref(shape), C.byref(cache), k, v, q, out, beacon_k, beacon_v,
                                        budget, live, ws, ws_bytes, stream)


def bc_diag_stream_read(src, nbytes, workgroups, mode, sink, stream):
    return load_diag().bc_diag_stream_read(src, nbytes, workgroups, mode, sink, stream)


def bc_sort_by_length(shape, cache, active, order, stream):
    return load().bc_sort_by_length(C.byref(shape), C.byref(cache), active, order, stream)


def bc_set_ratio(shape, cache, new_c, active, stream):
    return load().bc_set_ratio(C.byref(shape), C.byref(cache), new_c, active, stream)


def bc_prefill_workspace_bytes(shape, total_rows):
    return load().bc_prefill_workspace_bytes(C.byref(shape), total_rows)


def bc_prefill_attn_ws(shape, q, k, v, row_offsets, P, c, max_rows, total_rows, out, lse, workspace,
                       workspace_bytes, stream):
    return load().bc_prefill_attn_ws(C.byref(shape), q, k, v, row_offsets, P, c, max_rows, total_rows, out,
                                     lse, workspace, workspace_bytes, stream)


def bc_prefill_attn(shape, q, k, v, row_offsets, P, c, max_rows, out, lse, stream):
    return load().bc_prefill_attn(C.byref(shape), q, k, v, row_offsets, P, c, max_rows, out, lse,
                                  stream)


def bc_prefill_bwd_workspace_bytes(shape, total_rows):
    return load().bc_prefill_bwd_workspace_bytes(C.byref(shape), total_rows)


def bc_prefill_attn_bwd(shape, q, k, v, out, lse, dout, row_offsets, P, c, max_rows, total_rows, dq, dk,
                        dv, ws, ws_bytes, stream):
    return load().bc_prefill_attn_bwd(C.byref(shape), q, k, v, out, lse, dout, row_offsets, P, c,
                                      max_rows, total_rows, dq, dk, dv, ws, ws_bytes, stream)


def bc_topk_kl_loss(T, V, k, student_logits, logits_dtype, teacher_logits, teacher_idx, loss_per_token,
                    lse, loss_mean, stream):
    return load().bc_topk_kl_loss(T, V, k, student_logits, logits_dtype, teacher_logits, teacher_idx,
                                  loss_per_token, lse, loss_mean, stream)


def bc_topk_kl_loss_bwd(T, V, k, student_logits, logits_dtype, teacher_logits, teacher_idx, lse,
                        grad_scale, dlogits, stream):
    return load().bc_topk_kl_loss_bwd(T, V, k, student_logits, logits_dtype, teacher_logits,
                                      teacher_idx, lse, grad_scale, dlogits, stream)


def bc_tables_to_host(shape, cache, nb_host, w_host, err_host, stream):
    return load().bc_tables_to_host(C.byref(shape), C.byref(cache), nb_host, w_host, err_host, stream)


# ---------------------------------------------------------------------------
# Device-memory plumbing (torch tensors) around the calls above.
# ---------------------------------------------------------------------------
def _np_dtype_code(dtype: str) -> int:
    return BC_BF16 if dtype == "bf16" else BC_F32


def to_device(x, dtype: str, device):
    """NumPy fp32 values (exact in `dtype`) or a torch tensor -> device tensor in library format."""
    import torch
    if isinstance(x, torch.Tensor):
        return x
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        u = np.ascontiguousarray(x).view(np.uint32)
        if np.any(u & np.uint32(0xFFFF)):
            raise ValueError("values are not exactly representable in bf16")
        bits = (u >> np.uint32(16)).astype(np.uint16).view(np.int16)
        return torch.from_numpy(bits).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)


def _stream_ptr():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Runtime:
    """Owns slabs, tables and workspace of one batch of caches; calls the C ABI."""

    def __init__(self, B, Hq, Hkv, d, dtype, scale, P, c, cap, device):
        import torch
        load()
        self.torch = torch
        self.device = device
        self.dtype = dtype
        self.B, self.Hq, self.Hkv, self.d = int(B), int(Hq), int(Hkv), int(d)
        self.shape = bc_shape(self.B, self.Hq, self.Hkv, self.d, _np_dtype_code(dtype), float(scale))
        self.P_host = np.asarray(P, dtype=np.int32).copy()
        self.c_host = np.asarray(c, dtype=np.int32).copy()
        self.cap_host = np.asarray(cap, dtype=np.int32).copy()
        base = np.zeros(self.B, dtype=np.int64)
        base[1:] = np.cumsum(self.cap_host.astype(np.int64))[:-1]
        self.base_host = base
        total_entries = int(self.cap_host.astype(np.int64).sum())
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.elem_dtype = tdt
        n_elem = total_entries * self.Hkv * self.d
        self.k_slab = torch.empty(n_elem, dtype=tdt, device=device)
        self.v_slab = torch.empty(n_elem, dtype=tdt, device=device)
        self.k_slab.fill_(float("nan"))          # poison: reading an unwritten row shows up
        self.v_slab.fill_(float("nan"))
        self.base = torch.from_numpy(base).to(device)
        self.cap = torch.from_numpy(self.cap_host).to(device)
        self.P = torch.from_numpy(self.P_host).to(device)
        self.c = torch.from_numpy(self.c_host).to(device)
        self.nb = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.w = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.err = torch.zeros(1, dtype=torch.int32, device=device)
        self.max_cap = int(self.cap_host.max())
        self.cache = bc_cache(self.k_slab.data_ptr(), self.v_slab.data_ptr(), self.base.data_ptr(),
                              self.cap.data_ptr(), self.P.data_ptr(), self.c.data_ptr(),
                              self.nb.data_ptr(), self.w.data_ptr(), self.err.data_ptr(),
                              self.max_cap, None, 0, 0, 0, 0)
        # equal prompt lengths and capacities (slabs laid out back to back): tell the library, which
        # may then request prompt rows before it has read the tables
        if (self.P_host == self.P_host[0]).all() and (self.cap_host == self.cap_host[0]).all() \
                and 0 < int(self.P_host[0]) <= int(self.cap_host[0]):
            self.cache.uniform_P = int(self.P_host[0])
            self.cache.uniform_cap = int(self.cap_host[0])
        self.order = None
        self.ws_bytes = int(bc_decode_workspace_bytes(self.shape, self.max_cap))
        self.ws = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device=device)
        _check(bc_workspace_init(_ptr(self.ws), self.ws.numel(), _stream_ptr()))
        self.out = torch.empty(self.B, self.Hq, self.d, dtype=torch.float32, device=device)

    # -- helpers --------------------------------------------------------------
    def dev(self, x):
        return to_device(x, self.dtype, self.device)

    def mask(self, active):
        if active is None:
            return None
        if isinstance(active, self.torch.Tensor):
            return active
        return self.torch.from_numpy(np.asarray(active, dtype=np.uint8)).to(self.device)

    # -- calls ----------------------------------------------------------------
    def cache_init(self, prompts_k, prompts_v):
        torch = self.torch
        off = np.zeros(self.B + 1, dtype=np.int64)
        off[1:] = np.cumsum([len(p) for p in prompts_k])
        total = int(off[-1])
        if total:
            kp = self.dev(np.concatenate([np.asarray(p, np.float32) for p in prompts_k], axis=0))
            vp = self.dev(np.concatenate([np.asarray(p, np.float32) for p in prompts_v], axis=0))
        else:
            kp = vp = None
        offd = torch.from_numpy(off).to(self.device)
        _check(bc_cache_init(self.shape, self.cache, _ptr(kp), _ptr(vp), _ptr(offd), total,
                             _stream_ptr()))
        torch.cuda.current_stream().synchronize()     # inputs may be freed after this

    def cache_admit(self, admit, prompts_k, prompts_v, new_c=None, live=None):
        """admit: [B] 0/1; prompts_k/v: per slot [P, Hkv, d] arrays (ignored where admit is 0);
        new_c: [B] or None; live: uint8 device tensor [B] or None."""
        torch = self.torch
        admit = np.asarray(admit, dtype=np.uint8)
        spans = [len(prompts_k[s]) if admit[s] else 0 for s in range(self.B)]
        off = np.zeros(self.B + 1, dtype=np.int64)
        off[1:] = np.cumsum(spans)
        total = int(off[-1])
        rows = [s for s in range(self.B) if admit[s] and spans[s]]
        if total:
            kp = self.dev(np.concatenate([np.asarray(prompts_k[s], np.float32) for s in rows], axis=0))
            vp = self.dev(np.concatenate([np.asarray(prompts_v[s], np.float32) for s in rows], axis=0))
        else:
            kp = vp = None
        offd = torch.from_numpy(off).to(self.device)
        ad = torch.from_numpy(admit).to(self.device)
        ncd = None if new_c is None else torch.from_numpy(np.asarray(new_c, dtype=np.int32)).to(self.device)
        _check(bc_cache_admit(self.shape, self.cache, _ptr(kp), _ptr(vp), _ptr(offd), total, _ptr(ncd),
                              _ptr(ad), _ptr(live), _stream_ptr()))
        torch.cuda.current_stream().synchronize()
        for s in range(self.B):           # host mirror of P, used by resident()
            if admit[s] and spans[s] <= int(self.cap_host[s]):
                self.P_host[s] = spans[s]

    def append_kv(self, k, v, active=None, kind=BC_ROW_TOKEN):
        k, v, a = self.dev(k), self.dev(v), self.mask(active)
        _check(bc_append_kv(self.shape, self.cache, _ptr(k), _ptr(v), _ptr(a), kind, _stream_ptr()))

    def decode_attn(self, q, active=None, out=None):
        q, a = self.dev(q), self.mask(active)
        out = self.out if out is None else out
        _check(bc_decode_attn(self.shape, self.cache, _ptr(q), _ptr(out), _ptr(a), _ptr(self.ws),
                              self.ws_bytes, _stream_ptr()))
        return out

    def compress_evict(self, bk=None, bv=None, active=None, require_full_window=True):
        bk = None if bk is None else self.dev(bk)
        bv = None if bv is None else self.dev(bv)
        a = self.mask(active)
        _check(bc_compress_evict(self.shape, self.cache, _ptr(bk), _ptr(bv), _ptr(a),
                                 1 if require_full_window else 0, _stream_ptr()))

    def decode_step(self, k, v, q, bk=None, bv=None, active=None, out=None):
        k, v, q, a = self.dev(k), self.dev(v), self.dev(q), self.mask(active)
        bk = None if bk is None else self.dev(bk)
        bv = None if bv is None else self.dev(bv)
        out = self.out if out is None else out
        _check(bc_decode_step(self.shape, self.cache, _ptr(k), _ptr(v), _ptr(q), _ptr(out),
                              _ptr(bk), _ptr(bv), _ptr(a), _ptr(self.ws), self.ws_bytes,
                              _stream_ptr()))
        return out

    def decode_step_noalloc(self, k, v, q, bk=None, bv=None, active=None, out=None):
        """bc_decode_step on the library's own scratch array instead of this object's workspace."""
        k, v, q, a = self.dev(k), self.dev(v), self.dev(q), self.mask(active)
        bk = None if bk is None else self.dev(bk)
        bv = None if bv is None else self.dev(bv)
        out = self.out if out is None else out
        _check(bc_decode_step_noalloc(self.shape, self.cache, _ptr(k), _ptr(v), _ptr(q), _ptr(out),
                                      _ptr(bk), _ptr(bv), _ptr(a), _stream_ptr()))
        return out

    def beacon_step(self, k, v, q, active=None, out=None):
        k, v, q, a = self.dev(k), self.dev(v), self.dev(q), self.mask(active)
        out = self.out if out is None else out
        _check(bc_beacon_step(self.shape, self.cache, _ptr(k), _ptr(v), _ptr(q), _ptr(out), _ptr(a),
                              _ptr(self.ws), self.ws_bytes, _stream_ptr()))
        return out

    def decode_step_budget(self, k, v, q, bk, bv, budget, live, out=None):
        """budget: int32 device tensor [B]; live: uint8 device tensor [B] (read and updated)."""
        k, v, q = self.dev(k), self.dev(v), self.dev(q)
        bk = None if bk is None else self.dev(bk)
        bv = None if bv is None else self.dev(bv)
        out = self.out if out is None else out
        _check(bc_decode_step_budget(self.shape, self.cache, _ptr(k), _ptr(v), _ptr(q), _ptr(out),
                                     _ptr(bk), _ptr(bv), _ptr(budget), _ptr(live), _ptr(self.ws),
                                     self.ws_bytes, _stream_ptr()))
        return out

    def sort_by_length(self, active=None):
        """Refresh the dispatch order (longest resident sequence first) and attach it to the cache:
        large ragged batches then start their longest sequences first."""
        if self.order is None:
            self.order = self.torch.arange(self.B, dtype=self.torch.int32, device=self.device)
            self.cache.order = self.order.data_ptr()
        a = self.mask(active)
        _check(bc_sort_by_length(self.shape, self.cache, _ptr(a), _ptr(self.order), _stream_ptr()))

    def set_ratio(self, new_c, active=None):
        nc = self.torch.from_numpy(np.asarray(new_c, dtype=np.int32)).to(self.device)
        a = self.mask(active)
        _check(bc_set_ratio(self.shape, self.cache, _ptr(nc), _ptr(a), _stream_ptr()))
        self.torch.cuda.current_stream().synchronize()

    def tables(self):
        nb = np.empty(self.B, dtype=np.int32)
        w = np.empty(self.B, dtype=np.int32)
        err = np.empty(1, dtype=np.int32)
        _check(bc_tables_to_host(self.shape, self.cache, nb.ctypes.data_as(C.c_void_p),
                                 w.ctypes.data_as(C.c_void_p), err.ctypes.data_as(C.c_void_p),
                                 _stream_ptr()))
        return nb, w, int(err[0])

    def set_tables(self, nb, w):
        """Place the caches in a given state (benchmarks start mid-rollout)."""
        self.nb.copy_(self.torch.from_numpy(np.asarray(nb, dtype=np.int32)))
        self.w.copy_(self.torch.from_numpy(np.asarray(w, dtype=np.int32)))

    def resident(self, s, nb=None, w=None):
        """(K, V) [L, Hkv, d] fp32 NumPy copies of the resident rows of sequence s."""
        if nb is None:
            nbs, ws, _ = self.tables()
            nb, w = int(nbs[s]), int(ws[s])
        L = int(self.P_host[s]) + nb + w
        cap = int(self.cap_host[s])
        E = self.Hkv * self.d
        lo = int(self.base_host[s]) * E
        out = []
        for slab in (self.k_slab, self.v_slab):
            blk = slab[lo:lo + cap * E].view(self.Hkv, cap, self.d)[:, :L, :]
            out.append(blk.permute(1, 0, 2).float().cpu().numpy())
        return out[0], out[1]


def prefill_attn(q, k, v, row_offsets, P, c, Hq, Hkv, d, scale, want_lse=True, workspace=False):
    """bc_prefill_attn (or, workspace=True, bc_prefill_attn_ws) on device tensors.

    q [R, Hq, d], k, v [R, Hkv, d] bf16 device tensors (trajectories concatenated);
    row_offsets [B+1] int64, P, c [B] int32 (host arrays).  Returns (out fp32 [R,Hq,d], lse or None).
    """
    import torch
    load()
    dev = q.device
    row_offsets = np.asarray(row_offsets, dtype=np.int64)
    B = len(row_offsets) - 1
    shape = bc_shape(B, Hq, Hkv, d, BC_BF16, float(scale))
    offd = torch.from_numpy(row_offsets).to(dev)
    Pd = torch.from_numpy(np.asarray(P, dtype=np.int32)).to(dev)
    cd = torch.from_numpy(np.asarray(c, dtype=np.int32)).to(dev)
    R = int(row_offsets[-1])
    out = torch.empty(R, Hq, d, dtype=torch.float32, device=dev)
    lse = torch.empty(R, Hq, dtype=torch.float32, device=dev) if want_lse else None
    max_rows = int(np.diff(row_offsets).max())
    if workspace:
        nbytes = int(bc_prefill_workspace_bytes(shape, R))
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        _check(bc_prefill_attn_ws(shape, _ptr(q), _ptr(k), _ptr(v), _ptr(offd), _ptr(Pd), _ptr(cd), max_rows, R,
                                  _ptr(out), _ptr(lse), _ptr(ws), nbytes, _stream_ptr()))
    else:
        _check(bc_prefill_attn(shape, _ptr(q), _ptr(k), _ptr(v), _ptr(offd), _ptr(Pd), _ptr(cd), max_rows,
                               _ptr(out), _ptr(lse), _stream_ptr()))
    torch.cuda.current_stream().synchronize()      # offd/Pd/cd (and the workspace) may be freed after this
    return out, lse


def prefill_attn_bwd(q, k, v, out, lse, dout, row_offsets, P, c, Hq, Hkv, d, scale):
    """bc_prefill_attn_bwd on device tensors (see prefill_attn); returns (dq, dk, dv) fp32."""
    import torch
    load()
    dev = q.device
    row_offsets = np.asarray(row_offsets, dtype=np.int64)
    B = len(row_offsets) - 1
    R = int(row_offsets[-1])
    shape = bc_shape(B, Hq, Hkv, d, BC_BF16, float(scale))
    offd = torch.from_numpy(row_offsets).to(dev)
    Pd = torch.from_numpy(np.asarray(P, dtype=np.int32)).to(dev)
    cd = torch.from_numpy(np.asarray(c, dtype=np.int32)).to(dev)
    dq = torch.full((R, Hq, d), float("nan"), dtype=torch.float32, device=dev)
    dk = torch.full((R, Hkv, d), float("nan"), dtype=torch.float32, device=dev)
    dv = torch.full((R, Hkv, d), float("nan"), dtype=torch.float32, device=dev)
    ws_bytes = int(bc_prefill_bwd_workspace_bytes(shape, R))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    max_rows = int(np.diff(row_offsets).max())
    _check(bc_prefill_attn_bwd(shape, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout),
                               _ptr(offd), _ptr(Pd), _ptr(cd), max_rows, R, _ptr(dq), _ptr(dk), _ptr(dv),
                               _ptr(ws), ws_bytes, _stream_ptr()))
    torch.cuda.current_stream().synchronize()
    return dq, dk, dv


def _logits_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return BC_BF16
    if t.dtype == torch.float32:
        return BC_F32
    raise BcError("logits must be bf16 or fp32 device tensors")


def topk_kl_loss(student_logits, teacher_logits, teacher_idx):
    """bc_topk_kl_loss on device tensors: student_logits [T, V] bf16/fp32, teacher_logits [T, k]
    fp32, teacher_idx [T, k] int32.  Returns (loss_per_token [T], lse [T], loss_mean [1]) fp32."""
    import torch
    load()
    T, V = student_logits.shape
    k = teacher_logits.shape[1]
    dev = student_logits.device
    loss = torch.full((T,), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((T,), float("nan"), dtype=torch.float32, device=dev)
    mean = torch.full((1,), float("nan"), dtype=torch.float32, device=dev)
    _check(bc_topk_kl_loss(T, V, k, _ptr(student_logits), _logits_code(student_logits),
                           _ptr(teacher_logits), _ptr(teacher_idx), _ptr(loss), _ptr(lse), _ptr(mean),
                           _stream_ptr()))
    torch.cuda.current_stream().synchronize()
    return loss, lse, mean


def topk_kl_loss_bwd(student_logits, teacher_logits, teacher_idx, lse, grad_scale):
    """bc_topk_kl_loss_bwd on device tensors; returns dlogits [T, V] in the logits' dtype."""
    import torch
    load()
    T, V = student_logits.shape
    k = teacher_logits.shape[1]
    dz = torch.full_like(student_logits, float("nan"))
    _check(bc_topk_kl_loss_bwd(T, V, k, _ptr(student_logits), _logits_code(student_logits),
                               _ptr(teacher_logits), _ptr(teacher_idx), _ptr(lse), float(grad_scale),
                               _ptr(dz), _stream_ptr()))
    torch.cuda.current_stream().synchronize()
    return dz
