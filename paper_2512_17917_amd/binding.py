"""Thin ctypes binding of libkvr.so (declared in include/kvr.h).

Argument marshalling only: every function has the name and the argument order
of its C entry point, takes torch tensors where the C call takes device
pointers, checks dtype / device / contiguity / minimum size, and passes
`data_ptr()` plus the current torch HIP stream.  Nothing is computed here.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

KVR_OK = 0
KVR_ERR_INVALID_ARG = -1
KVR_ERR_UNSUPPORTED = -2
KVR_ERR_WORKSPACE_TOO_SMALL = -3
KVR_ERR_HIP = -4
KVR_F32, KVR_BF16 = 0, 1
KVR_MEDIAN_MIDMEAN, KVR_MEDIAN_LOWER = 0, 1
KVR_OP_SELECT, KVR_OP_ENCODE, KVR_OP_RECONSTRUCT, KVR_OP_ATTEND = 0, 1, 2, 3
KVR_MAX_ROWS = 8
KVR_HEAD_DIM = 128

_ERR_NAMES = {-1: "KVR_ERR_INVALID_ARG", -2: "KVR_ERR_UNSUPPORTED",
              -3: "KVR_ERR_WORKSPACE_TOO_SMALL", -4: "KVR_ERR_HIP"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvr.so")

EXPORTS = ["kvr_version", "kvr_last_hip_error", "kvr_recent_size", "kvr_hash_params_from_seed", "kvr_hash_host",
           "kvr_workspace_size", "kvr_append", "kvr_select", "kvr_encode", "kvr_step_update",
           "kvr_swap_back", "kvr_reconstruct", "kvr_attend_decode", "kvr_attend_decode_static",
           "kvr_attend_multi_workspace_size", "kvr_attend_multi"]
KVR_STATIC_SCRATCH_BYTES = 80 << 20


class KvrError(RuntimeError):
    def __init__(self, fn, code, hip=0):
        self.code = code
        self.hip = hip
        super().__init__(f"{fn} failed: {_ERR_NAMES.get(code, code)}" + (f" (hipError {hip})" if hip else ""))


class kvr_desc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("r", C.c_int32), ("w", C.c_int32), ("dtype", C.c_int32),
                ("sign_mask", C.c_int32), ("median_mode", C.c_int32), ("softmax_scale", C.c_float),
                ("hash_params", (C.c_uint64 * 4) * KVR_MAX_ROWS)]


class kvr_attend_opts(C.Structure):
    _fields_ = [("side_stream", C.c_void_p), ("fork_event", C.c_void_p), ("join_event", C.c_void_p),
                ("prof_start", C.c_void_p), ("prof_stop", C.c_void_p)]


_lib = None
_hip = None


def hip() -> C.CDLL:
    """The HIP runtime, for the few raw handles the C ABI takes (events)."""
    global _hip
    if _hip is None:
        h = C.CDLL("libamdhip64.so")
        h.hipEventCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        h.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        h.hipEventDestroy.argtypes = [C.c_void_p]
        _hip = h
    return _hip


def event_create(timing: bool) -> C.c_void_p:
    ev = C.c_void_p()
    rc = hip().hipEventCreateWithFlags(C.byref(ev), 0 if timing else 2)      # 2 = hipEventDisableTiming
    if rc != 0:
        raise RuntimeError(f"hipEventCreateWithFlags failed: {rc}")
    return ev


def event_elapsed_ms(a, b) -> float:
    ms = C.c_float()
    rc = hip().hipEventElapsedTime(C.byref(ms), a, b)
    if rc != 0:
        raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
    return ms.value


class SideStream:
    """A second stream (default priority) and the fork / join events that a caller
    lends to kvr_attend_decode so that its two main kernels can run side by side.
    Plumbing only.  One object serves any number of calls that are ordered on one
    stream."""

    def __init__(self, device="cuda"):
        self.stream = torch.cuda.Stream(device=device)
        self.fork = event_create(False)
        self.join = event_create(False)

    def opts(self, prof_start=None, prof_stop=None) -> "kvr_attend_opts":
        return kvr_attend_opts(self.stream.cuda_stream, self.fork, self.join, prof_start, prof_stop)

    def __del__(self):
        try:
            hip().hipEventDestroy(self.fork)
            hip().hipEventDestroy(self.join)
        except Exception:
            pass


def lib() -> C.CDLL:
    """Load libkvr.so (built by paper_2512_17917_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2512_17917_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        dp = C.POINTER(kvr_desc)
        L.kvr_version.restype = C.c_char_p
        L.kvr_version.argtypes = []
        L.kvr_last_hip_error.restype = i32
        L.kvr_last_hip_error.argtypes = []
        L.kvr_recent_size.restype = i32
        L.kvr_recent_size.argtypes = [i32, i32, i32]
        L.kvr_hash_params_from_seed.restype = i32
        L.kvr_hash_params_from_seed.argtypes = [C.c_uint64, i32, C.POINTER(C.c_uint64)]
        L.kvr_hash_host.restype = i32
        L.kvr_hash_host.argtypes = [dp, i32, C.POINTER(i32), C.POINTER(i32)]
        L.kvr_workspace_size.restype = i32
        L.kvr_workspace_size.argtypes = [dp, i32, i64, i64, C.POINTER(sz)]
        L.kvr_append.restype = i32
        L.kvr_append.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
        L.kvr_select.restype = i32
        L.kvr_select.argtypes = [dp, vp, i64, vp, i32, vp, i32, i32, vp, vp, vp, i32, vp, vp, i32,
                                 vp, sz, vp]
        L.kvr_encode.restype = i32
        L.kvr_encode.argtypes = [dp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.kvr_step_update.restype = i32
        L.kvr_step_update.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, i64, i32, i32, vp, vp, vp, i32,
                                      vp, vp, i32, vp, vp, vp]
        L.kvr_swap_back.restype = i32
        L.kvr_swap_back.argtypes = [dp, vp, i64, vp, vp, vp, i32, vp, i32, C.c_float, i32, vp, vp, vp, vp, i32,
                                    vp, vp, vp]
        L.kvr_reconstruct.restype = i32
        L.kvr_reconstruct.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp]
        L.kvr_attend_decode.restype = i32
        L.kvr_attend_decode.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, i64,
                                        vp, sz, C.POINTER(kvr_attend_opts), vp]
        L.kvr_attend_decode_static.restype = i32
        L.kvr_attend_decode_static.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, i64,
                                               C.POINTER(kvr_attend_opts), vp]
        L.kvr_attend_multi_workspace_size.restype = i32
        L.kvr_attend_multi_workspace_size.argtypes = [dp, i32, i64, i64, C.POINTER(sz)]
        L.kvr_attend_multi.restype = i32
        L.kvr_attend_multi.argtypes = [dp, vp, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, i64,
                                       vp, sz, vp]
        _lib = L
    return _lib


def _check(fn, rc):
    if rc != KVR_OK:
        raise KvrError(fn, rc, lib().kvr_last_hip_error() if rc == KVR_ERR_HIP else 0)


def make_desc(batch, n_q_heads, n_kv_heads, r, w, dtype, *, seed=None, hash_params=None,
              sign_mask=2, median_mode=KVR_MEDIAN_MIDMEAN, softmax_scale=None, head_dim=KVR_HEAD_DIM):
    """Fill a kvr_desc.  dtype: torch.float32 / torch.bfloat16 or KVR_F32 / KVR_BF16.
    hash_params: r rows of (a, b, c, d), or derived from `seed` by the library."""
    d = kvr_desc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = batch, n_q_heads, n_kv_heads, head_dim
    d.r, d.w = r, w
    if dtype in (torch.float32, KVR_F32):
        d.dtype = KVR_F32
    elif dtype in (torch.bfloat16, KVR_BF16):
        d.dtype = KVR_BF16
    else:
        raise ValueError(f"unsupported dtype {dtype}")
    d.sign_mask, d.median_mode = sign_mask, median_mode
    d.softmax_scale = (head_dim ** -0.5) if softmax_scale is None else softmax_scale
    if hash_params is None:
        hash_params = kvr_hash_params_from_seed(0 if seed is None else seed, r)
    for i, row in enumerate(hash_params):
        for k in range(4):
            d.hash_params[i][k] = int(row[k]) & ((1 << 64) - 1)
    return d


def desc_hash_params(d: kvr_desc):
    return [tuple(int(d.hash_params[i][k]) for k in range(4)) for i in range(d.r)]


def _torch_dtype(d: kvr_desc):
    return torch.float32 if d.dtype == KVR_F32 else torch.bfloat16


def _ptr(t, dtype, min_numel, name, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise ValueError(f"{name} is required")
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if t.numel() < min_numel:
        raise ValueError(f"{name}: {t.numel()} elements, need at least {min_numel}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    if not (isinstance(ws, torch.Tensor) and ws.is_cuda and ws.is_contiguous()):
        raise ValueError("ws must be a contiguous device tensor")
    return ws.data_ptr(), ws.numel() * ws.element_size()


# ---------------------------------------------------------------------------
def kvr_version() -> str:
    return lib().kvr_version().decode()


def kvr_recent_size(r_size: int, r_budget: int, slack: int) -> int:
    rc = lib().kvr_recent_size(r_size, r_budget, slack)
    if rc < 0:
        raise KvrError("kvr_recent_size", rc)
    return int(rc)


def kvr_hash_params_from_seed(seed: int, r: int):
    buf = (C.c_uint64 * (4 * r))()
    _check("kvr_hash_params_from_seed", lib().kvr_hash_params_from_seed(seed & ((1 << 64) - 1), r, buf))
    return [tuple(int(buf[i * 4 + k]) for k in range(4)) for i in range(r)]


def kvr_hash_host(desc: kvr_desc, J: int):
    b = (C.c_int32 * KVR_MAX_ROWS)()
    s = (C.c_int32 * KVR_MAX_ROWS)()
    _check("kvr_hash_host", lib().kvr_hash_host(C.byref(desc), J, b, s))
    return [int(b[i]) for i in range(desc.r)], [int(s[i]) for i in range(desc.r)]


def kvr_workspace_size(desc: kvr_desc, op: int, n_a: int, n_b: int = 0) -> int:
    out = C.c_size_t(0)
    _check("kvr_workspace_size", lib().kvr_workspace_size(C.byref(desc), op, n_a, n_b, C.byref(out)))
    return int(out.value)


def alloc_workspace(desc: kvr_desc, op: int, n_a: int, n_b: int = 0, device="cuda") -> torch.Tensor:
    n = kvr_workspace_size(desc, op, n_a, n_b)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def kvr_append(desc, k_new, v_new, n_ctx, k_ret, v_ret, ret_pos, ret_cap, out_slot=None):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    rc = lib().kvr_append(
        C.byref(desc), _ptr(k_new, dt, U * D, "k_new"), _ptr(v_new, dt, U * D, "v_new"),
        _ptr(n_ctx, torch.int32, desc.batch, "n_ctx"),
        _ptr(k_ret, dt, U * ret_cap * D, "k_ret"), _ptr(v_ret, dt, U * ret_cap * D, "v_ret"),
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos"), ret_cap,
        _ptr(out_slot, torch.int32, U, "out_slot", True), _stream())
    _check("kvr_append", rc)


def kvr_select(desc, scores, n_cap, ret_pos, ret_cap, n_ctx, n_recent, k_candidate,
               evict_slot, evict_pos, n_evict, evict_cap, vague_pos, n_vague, vague_cap, ws=None):
    U = desc.batch * desc.n_kv_heads
    wp, wb = _ws(ws)
    rc = lib().kvr_select(
        C.byref(desc), _ptr(scores, torch.float32, U * n_cap, "scores"), n_cap,
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos"), ret_cap,
        _ptr(n_ctx, torch.int32, desc.batch, "n_ctx"), n_recent, k_candidate,
        _ptr(evict_slot, torch.int32, U * evict_cap, "evict_slot"),
        _ptr(evict_pos, torch.int32, U * evict_cap, "evict_pos"),
        _ptr(n_evict, torch.int32, U, "n_evict"), evict_cap,
        _ptr(vague_pos, torch.int32, U * vague_cap, "vague_pos", True),
        _ptr(n_vague, torch.int32, U, "n_vague", True), vague_cap, wp, wb, _stream())
    _check("kvr_select", rc)


def kvr_encode(desc, k_src, v_src, src_rows, src_slot, tok_pos, count, cap, sketch_k, sketch_v,
               out_bucket=None, out_sign=None, ws=None):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    wp, wb = _ws(ws)
    rc = lib().kvr_encode(
        C.byref(desc), _ptr(k_src, dt, U * src_rows * D, "k_src"), _ptr(v_src, dt, U * src_rows * D, "v_src"),
        src_rows, _ptr(src_slot, torch.int32, U * cap, "src_slot"),
        _ptr(tok_pos, torch.int32, U * cap, "tok_pos"), _ptr(count, torch.int32, U, "count"), cap,
        _ptr(sketch_k, dt, U * S, "sketch_k"), _ptr(sketch_v, dt, U * S, "sketch_v"),
        _ptr(out_bucket, torch.int32, U * cap * desc.r, "out_bucket", True),
        _ptr(out_sign, torch.uint8, U * cap, "out_sign", True), wp, wb, _stream())
    _check("kvr_encode", rc)


def kvr_step_update(desc, k_new, v_new, n_ctx, k_ret, v_ret, ret_pos, ret_cap, scores, n_cap, n_recent,
                    k_candidate, evict_slot, evict_pos, n_evict, evict_cap, vague_pos, n_vague, vague_cap,
                    sketch_k, sketch_v):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    rc = lib().kvr_step_update(
        C.byref(desc), _ptr(k_new, dt, U * D, "k_new"), _ptr(v_new, dt, U * D, "v_new"),
        _ptr(n_ctx, torch.int32, desc.batch, "n_ctx"),
        _ptr(k_ret, dt, U * ret_cap * D, "k_ret"), _ptr(v_ret, dt, U * ret_cap * D, "v_ret"),
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos"), ret_cap,
        _ptr(scores, torch.float32, U * n_cap, "scores"), n_cap, n_recent, k_candidate,
        _ptr(evict_slot, torch.int32, U * evict_cap, "evict_slot"),
        _ptr(evict_pos, torch.int32, U * evict_cap, "evict_pos"),
        _ptr(n_evict, torch.int32, U, "n_evict"), evict_cap,
        _ptr(vague_pos, torch.int32, U * vague_cap, "vague_pos", True),
        _ptr(n_vague, torch.int32, U, "n_vague", True), vague_cap,
        _ptr(sketch_k, dt, U * S, "sketch_k"), _ptr(sketch_v, dt, U * S, "sketch_v"), _stream())
    _check("kvr_step_update", rc)


def kvr_swap_back(desc, scores, n_cap, k_ret, v_ret, ret_pos, ret_cap, n_ctx, n_recent, replace_rate,
                  max_swaps, sketch_k, sketch_v, vague_pos, n_vague, vague_cap, n_swapped=None, swap_log=None):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    rc = lib().kvr_swap_back(
        C.byref(desc), _ptr(scores, torch.float32, U * n_cap, "scores"), n_cap,
        _ptr(k_ret, dt, U * ret_cap * D, "k_ret"), _ptr(v_ret, dt, U * ret_cap * D, "v_ret"),
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos"), ret_cap,
        _ptr(n_ctx, torch.int32, desc.batch, "n_ctx"), n_recent, C.c_float(replace_rate), max_swaps,
        _ptr(sketch_k, dt, U * S, "sketch_k"), _ptr(sketch_v, dt, U * S, "sketch_v"),
        _ptr(vague_pos, torch.int32, U * vague_cap, "vague_pos"), _ptr(n_vague, torch.int32, U, "n_vague"),
        vague_cap, _ptr(n_swapped, torch.int32, U, "n_swapped", True),
        _ptr(swap_log, torch.int32, U * max(max_swaps, 1) * 2, "swap_log", True), _stream())
    _check("kvr_swap_back", rc)


def kvr_reconstruct(desc, sketch_k, sketch_v, tok_pos, count, cap, k_out, v_out):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    rc = lib().kvr_reconstruct(
        C.byref(desc), _ptr(sketch_k, dt, U * S, "sketch_k"), _ptr(sketch_v, dt, U * S, "sketch_v"),
        _ptr(tok_pos, torch.int32, U * cap, "tok_pos"), _ptr(count, torch.int32, U, "count"), cap,
        _ptr(k_out, dt, U * cap * D, "k_out"), _ptr(v_out, dt, U * cap * D, "v_out"), _stream())
    _check("kvr_reconstruct", rc)


def kvr_attend_decode(desc, q, k_ret, v_ret, ret_pos, ret_cap, sketch_k, sketch_v, vague_pos, n_vague,
                      vague_cap, out, scores, n_cap, ws, opts=None):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    wp, wb = _ws(ws)
    rc = lib().kvr_attend_decode(
        C.byref(desc), _ptr(q, dt, desc.batch * desc.n_q_heads * D, "q"),
        _ptr(k_ret, dt, U * ret_cap * D, "k_ret"), _ptr(v_ret, dt, U * ret_cap * D, "v_ret"),
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos", True), ret_cap,
        _ptr(sketch_k, dt, U * S, "sketch_k", True), _ptr(sketch_v, dt, U * S, "sketch_v", True),
        _ptr(vague_pos, torch.int32, U * vague_cap, "vague_pos", True),
        _ptr(n_vague, torch.int32, U, "n_vague", True), vague_cap,
        _ptr(out, torch.float32, desc.batch * desc.n_q_heads * D, "out"),
        _ptr(scores, torch.float32, U * n_cap, "scores", True), n_cap, wp, wb,
        C.byref(opts) if opts is not None else None, _stream())
    _check("kvr_attend_decode", rc)


def kvr_attend_decode_static(desc, q, k_ret, v_ret, ret_pos, ret_cap, sketch_k, sketch_v, vague_pos, n_vague,
                             vague_cap, out, scores, n_cap, opts=None):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    rc = lib().kvr_attend_decode_static(
        C.byref(desc), _ptr(q, dt, desc.batch * desc.n_q_heads * D, "q"),
        _ptr(k_ret, dt, U * ret_cap * D, "k_ret"), _ptr(v_ret, dt, U * ret_cap * D, "v_ret"),
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos", True), ret_cap,
        _ptr(sketch_k, dt, U * S, "sketch_k", True), _ptr(sketch_v, dt, U * S, "sketch_v", True),
        _ptr(vague_pos, torch.int32, U * vague_cap, "vague_pos", True),
        _ptr(n_vague, torch.int32, U, "n_vague", True), vague_cap,
        _ptr(out, torch.float32, desc.batch * desc.n_q_heads * D, "out"),
        _ptr(scores, torch.float32, U * n_cap, "scores", True), n_cap,
        C.byref(opts) if opts is not None else None, _stream())
    _check("kvr_attend_decode_static", rc)


def kvr_attend_multi_workspace_size(desc, n_q, ret_cap, vague_cap) -> int:
    n = C.c_size_t(0)
    _check("kvr_attend_multi_workspace_size",
           lib().kvr_attend_multi_workspace_size(C.byref(desc), n_q, ret_cap, vague_cap, C.byref(n)))
    return n.value


def kvr_attend_multi(desc, q, n_q, n_ctx, k_ret, v_ret, ret_pos, ret_cap, sketch_k, sketch_v, vague_pos, n_vague,
                     vague_cap, out, scores, n_cap, ws):
    U, D, dt = desc.batch * desc.n_kv_heads, desc.head_dim, _torch_dtype(desc)
    S = desc.r * desc.w * D
    wp, wb = _ws(ws)
    rc = lib().kvr_attend_multi(
        C.byref(desc), _ptr(q, dt, desc.batch * n_q * desc.n_q_heads * D, "q"), n_q,
        _ptr(n_ctx, torch.int32, desc.batch, "n_ctx"),
        _ptr(k_ret, dt, U * ret_cap * D, "k_ret"), _ptr(v_ret, dt, U * ret_cap * D, "v_ret"),
        _ptr(ret_pos, torch.int32, U * ret_cap, "ret_pos"), ret_cap,
        _ptr(sketch_k, dt, U * S, "sketch_k", True), _ptr(sketch_v, dt, U * S, "sketch_v", True),
        _ptr(vague_pos, torch.int32, U * vague_cap, "vague_pos", True),
        _ptr(n_vague, torch.int32, U, "n_vague", True), vague_cap,
        _ptr(out, torch.float32, desc.batch * n_q * desc.n_q_heads * D, "out"),
        _ptr(scores, torch.float32, U * n_cap, "scores", True), n_cap, wp, wb, _stream())
    _check("kvr_attend_multi", rc)
