"""Python binding over libhmi.so (argument marshalling only).

Every step of the mixed-tenant layer forward runs inside the HIP library; this module
turns torch tensors / numpy arrays into raw pointers and forwards the call under the
same names as the C ABI (include/hmi.h).  There is no CPU fallback: importing the
binding without the built library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
# Before the library is loaded: torch ships its own HIP runtime, and the device buffers and streams the calls
# below receive come from it.  The library has to bind to that same runtime; loaded first, it would bring in the
# system's, and the second runtime to initialise in a process finds no device.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("HMI_LIB_PATH") or os.path.join(_HERE, "libhmi.so")  # override: alternative builds

HMI_OK, HMI_ERR_ARG, HMI_ERR_OOM, HMI_ERR_TENANT, HMI_ERR_SHAPE, HMI_ERR_CAPACITY, HMI_ERR_DEVICE = \
    0, -1, -2, -3, -4, -5, -6
HMI_F32, HMI_BF16 = 0, 1
HMI_BLOCK_FFN, HMI_BLOCK_ENC_POSTLN, HMI_BLOCK_DEC_PRELN, HMI_BLOCK_ADAPTER, HMI_BLOCK_ENC_ADAPTER, HMI_BLOCK_DEC_ADAPTER = 0, 1, 2, 3, 4, 5

EXPORTS = ["hmi_pool_create", "hmi_pool_load_tenant", "hmi_pool_alias_tenant", "hmi_pool_load_shared", "hmi_pool_load_head", "hmi_head_forward",
           "hmi_kv_create", "hmi_prefill", "hmi_decode_step", "hmi_plot_aggregate", "hmi_layer_forward", "hmi_layer_forward_static", "hmi_stack_forward", "hmi_stack_forward_f32",
           "hmi_get_route",
           "hmi_pool_prefetch", "hmi_pool_stats", "hmi_pool_profile", "hmi_pool_profile_read", "hmi_pool_image_bytes", "hmi_last_error",
           "hmi_pool_destroy",
           "hmi_queue_create", "hmi_queue_push", "hmi_queue_run", "hmi_queue_fetch", "hmi_queue_waiting",
           "hmi_queue_last_error", "hmi_queue_destroy"]


class hmi_pool_config_t(C.Structure):
    _fields_ = [("block", C.c_int32), ("dtype", C.c_int32), ("d_model", C.c_int32),
                ("d_ff", C.c_int32), ("n_heads", C.c_int32), ("n_layers", C.c_int32),
                ("max_tenants", C.c_int32), ("hbm_slots", C.c_int32), ("host_tier", C.c_int32),
                ("max_requests", C.c_int32), ("max_tokens", C.c_int32), ("ln_eps", C.c_float),
                ("device", C.c_int32), ("compute_stream", C.c_void_p), ("adapter_rank", C.c_int32), ("max_classes", C.c_int32)]


class HmiError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libhmi error {code}: {msg}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python paper_2504_17449_amd/build.py` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
    pi32 = C.POINTER(C.c_int32)
    lib.hmi_pool_create.argtypes = [C.POINTER(hmi_pool_config_t), C.POINTER(vp)]
    lib.hmi_pool_create.restype = i32
    lib.hmi_pool_load_tenant.argtypes = [vp, i32, i32, C.POINTER(vp), i32]
    lib.hmi_pool_load_tenant.restype = i32
    lib.hmi_pool_alias_tenant.argtypes = [vp, i32, i32]
    lib.hmi_pool_alias_tenant.restype = i32
    lib.hmi_pool_load_shared.argtypes = [vp, i32, C.POINTER(vp), i32]
    lib.hmi_pool_load_shared.restype = i32
    lib.hmi_pool_load_head.argtypes = [vp, i32, vp, vp, i32, i32]
    lib.hmi_pool_load_head.restype = i32
    lib.hmi_head_forward.argtypes = [vp, vp, vp, vp]
    lib.hmi_head_forward.restype = i32
    lib.hmi_plot_aggregate.argtypes = [vp, vp, i32, vp, pi32, i32, vp]
    lib.hmi_plot_aggregate.restype = i32
    lib.hmi_kv_create.argtypes = [vp, i32, i32]
    lib.hmi_kv_create.restype = i32
    lib.hmi_prefill.argtypes = [vp, i32, i32, vp, vp, pi32, pi32, pi32, i32]
    lib.hmi_prefill.restype = i32
    lib.hmi_decode_step.argtypes = [vp, i32, i32, vp, vp, pi32, pi32, i32]
    lib.hmi_decode_step.restype = i32
    lib.hmi_layer_forward.argtypes = [vp, i32, vp, vp, pi32, pi32, i32]
    lib.hmi_layer_forward.restype = i32
    lib.hmi_layer_forward_static.argtypes = [vp, i32, vp, vp, pi32, pi32, i32]
    lib.hmi_layer_forward_static.restype = i32
    lib.hmi_stack_forward.argtypes = [vp, i32, i32, vp, vp, pi32, pi32, i32]
    lib.hmi_stack_forward.restype = i32
    lib.hmi_stack_forward_f32.argtypes = [vp, i32, i32, vp, vp, pi32, pi32, i32]
    lib.hmi_stack_forward_f32.restype = i32
    lib.hmi_get_route.argtypes = [vp, pi32, pi32, pi32, pi32, pi32]
    lib.hmi_get_route.restype = i32
    lib.hmi_pool_prefetch.argtypes = [vp, i32, pi32, i32]
    lib.hmi_pool_prefetch.restype = i32
    lib.hmi_pool_stats.argtypes = [vp] + [C.POINTER(i64)] * 4
    lib.hmi_pool_stats.restype = i32
    lib.hmi_pool_profile.argtypes = [vp, i32]
    lib.hmi_pool_profile.restype = i32
    lib.hmi_pool_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.hmi_pool_profile_read.restype = i32
    lib.hmi_pool_image_bytes.argtypes = [vp]
    lib.hmi_pool_image_bytes.restype = i64
    lib.hmi_last_error.argtypes = [vp]
    lib.hmi_last_error.restype = C.c_char_p
    lib.hmi_pool_destroy.argtypes = [vp]
    lib.hmi_pool_destroy.restype = i32
    lib.hmi_queue_create.argtypes = [vp, i32, i32, i32, C.POINTER(vp)]
    lib.hmi_queue_create.restype = i32
    lib.hmi_queue_push.argtypes = [vp, i32, i32, vp, C.POINTER(i64)]
    lib.hmi_queue_push.restype = i32
    lib.hmi_queue_run.argtypes = [vp, C.POINTER(i64), pi32]
    lib.hmi_queue_run.restype = i32
    lib.hmi_queue_fetch.argtypes = [vp, i64, vp]
    lib.hmi_queue_fetch.restype = i32
    lib.hmi_queue_waiting.argtypes = [vp]
    lib.hmi_queue_waiting.restype = i32
    lib.hmi_queue_last_error.argtypes = [vp]
    lib.hmi_queue_last_error.restype = C.c_char_p
    lib.hmi_queue_destroy.argtypes = [vp]
    lib.hmi_queue_destroy.restype = i32
    return lib


lib = _load()


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _p32(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


# ---------------------------------------------------------------- same names as the C ABI

def hmi_last_error(pool: Optional[int]) -> str:
    return (lib.hmi_last_error(pool) or b"").decode()


def hmi_pool_create(*, block: int, dtype: int, d_model: int, d_ff: int, n_heads: int = 0,
                    n_layers: int = 1, max_tenants: int, hbm_slots: Optional[int] = None,
                    host_tier: bool = False, max_requests: int, max_tokens: int,
                    ln_eps: float = 1e-12, device: int = 0, compute_stream: int = 0, adapter_rank: int = 0,
                    max_classes: int = 0):
    """-> (status, pool handle or None).  compute_stream: raw hipStream_t (torch's
    ``torch.cuda.current_stream().cuda_stream``), 0 = default stream."""
    cfg = hmi_pool_config_t(block, dtype, d_model, d_ff, n_heads, n_layers, max_tenants,
                            max_tenants if hbm_slots is None else hbm_slots, int(host_tier),
                            max_requests, max_tokens, ln_eps, device, compute_stream or None, adapter_rank, max_classes)
    out = C.c_void_p()
    rc = lib.hmi_pool_create(C.byref(cfg), C.byref(out))
    return rc, (out.value if rc == HMI_OK else None)


def hmi_pool_load_tenant(pool: int, tenant_id: int, layer: int, tensors: Sequence[np.ndarray]) -> int:
    """tensors: host numpy arrays in canonical order, already in the pool's storage dtype
    (uint16 bf16 bit patterns or float32), C-contiguous."""
    keep = [np.ascontiguousarray(t) for t in tensors]
    arr = (C.c_void_p * len(keep))(*[t.ctypes.data for t in keep])
    return lib.hmi_pool_load_tenant(pool, tenant_id, layer, arr, len(keep))


def hmi_pool_alias_tenant(pool: int, tenant_id: int, source_tenant: int) -> int:
    return lib.hmi_pool_alias_tenant(pool, tenant_id, source_tenant)


def hmi_pool_load_shared(pool: int, layer: int, tensors: Sequence[np.ndarray]) -> int:
    """tensors: the shared layer's host arrays in canonical order, pool storage dtype."""
    keep = [np.ascontiguousarray(t) for t in tensors]
    arr = (C.c_void_p * len(keep))(*[t.ctypes.data for t in keep])
    return lib.hmi_pool_load_shared(pool, layer, arr, len(keep))


def hmi_pool_load_head(pool: int, tenant_id: int, w: np.ndarray, b: np.ndarray, per_token: bool) -> int:
    """w [n_classes, d], b [n_classes]: host arrays in the pool's storage dtype."""
    w, b = np.ascontiguousarray(w), np.ascontiguousarray(b)
    return lib.hmi_pool_load_head(pool, tenant_id, w.ctypes.data, b.ctypes.data, w.shape[0], int(per_token))


def hmi_head_forward(pool: int, h_ptr: int, scores_ptr: int, labels_ptr: int) -> int:
    """Device addresses; scores_ptr may be 0."""
    return lib.hmi_head_forward(pool, h_ptr, scores_ptr or None, labels_ptr)


def hmi_plot_aggregate(pool: int, table_ptr: int, n_entries: int, frag_ids_ptr: int, seq_lens, x_ptr: int) -> int:
    """table_ptr / frag_ids_ptr / x_ptr: device addresses; seq_lens: host ints."""
    lens = _i32(seq_lens)
    return lib.hmi_plot_aggregate(pool, table_ptr, n_entries, frag_ids_ptr, _p32(lens), lens.shape[0], x_ptr)


def hmi_kv_create(pool: int, max_seqs: int, max_len: int) -> int:
    return lib.hmi_kv_create(pool, max_seqs, max_len)


def hmi_prefill(pool: int, layer_begin: int, layer_end: int, x_ptr: int, y_ptr: int, tenant_ids, seq_lens,
                seq_slots) -> int:
    ids, lens, slots = _i32(tenant_ids), _i32(seq_lens), _i32(seq_slots)
    if not (ids.shape == lens.shape == slots.shape) or ids.ndim != 1:
        raise ValueError("tenant_ids, seq_lens and seq_slots must be 1-D and of equal length")
    return lib.hmi_prefill(pool, layer_begin, layer_end, x_ptr, y_ptr, _p32(ids), _p32(lens), _p32(slots), ids.shape[0])


def hmi_decode_step(pool: int, layer_begin: int, layer_end: int, x_ptr: int, y_ptr: int, tenant_ids, seq_slots) -> int:
    ids, slots = _i32(tenant_ids), _i32(seq_slots)
    if ids.shape != slots.shape or ids.ndim != 1:
        raise ValueError("tenant_ids and seq_slots must be 1-D and of equal length")
    return lib.hmi_decode_step(pool, layer_begin, layer_end, x_ptr, y_ptr, _p32(ids), _p32(slots), ids.shape[0])


def hmi_layer_forward(pool: int, layer: int, x_ptr: int, y_ptr: int, tenant_ids, seq_lens) -> int:
    """x_ptr / y_ptr: device addresses (tensor.data_ptr()); tenant_ids / seq_lens: host ints."""
    ids, lens = _i32(tenant_ids), _i32(seq_lens)
    if ids.shape != lens.shape or ids.ndim != 1:
        raise ValueError("tenant_ids and seq_lens must be 1-D and of equal length")
    return lib.hmi_layer_forward(pool, layer, x_ptr, y_ptr, _p32(ids), _p32(lens), ids.shape[0])


def hmi_layer_forward_static(pool: int, layer: int, x_ptr: int, y_ptr: int, tenant_ids, seq_lens) -> int:
    """hmi_layer_forward through the library's static routing arrays (allocates nothing)."""
    ids, lens = _i32(tenant_ids), _i32(seq_lens)
    if ids.shape != lens.shape or ids.ndim != 1:
        raise ValueError("tenant_ids and seq_lens must be 1-D and of equal length")
    return lib.hmi_layer_forward_static(pool, layer, x_ptr, y_ptr, _p32(ids), _p32(lens), ids.shape[0])


def hmi_stack_forward(pool: int, layer_begin: int, layer_end: int, x_ptr: int, y_ptr: int,
                      tenant_ids, seq_lens) -> int:
    ids, lens = _i32(tenant_ids), _i32(seq_lens)
    if ids.shape != lens.shape or ids.ndim != 1:
        raise ValueError("tenant_ids and seq_lens must be 1-D and of equal length")
    return lib.hmi_stack_forward(pool, layer_begin, layer_end, x_ptr, y_ptr, _p32(ids), _p32(lens),
                                 ids.shape[0])


def hmi_stack_forward_f32(pool: int, layer_begin: int, layer_end: int, x_ptr: int, y_ptr: int,
                          tenant_ids, seq_lens) -> int:
    ids, lens = _i32(tenant_ids), _i32(seq_lens)
    if ids.shape != lens.shape or ids.ndim != 1:
        raise ValueError("tenant_ids and seq_lens must be 1-D and of equal length")
    return lib.hmi_stack_forward_f32(pool, layer_begin, layer_end, x_ptr, y_ptr, _p32(ids), _p32(lens),
                                     ids.shape[0])


def hmi_get_route(pool: int, max_requests: int):
    perm = np.zeros(max_requests, np.int32)
    seg_tenant = np.zeros(max_requests, np.int32)
    seg_req_off = np.zeros(max_requests + 1, np.int32)
    seg_tok_off = np.zeros(max_requests + 1, np.int32)
    G = C.c_int32(0)
    rc = lib.hmi_get_route(pool, _p32(perm), _p32(seg_tenant), _p32(seg_req_off), _p32(seg_tok_off),
                           C.byref(G))
    g = G.value
    return rc, {"perm": perm, "seg_tenant": seg_tenant[:g], "seg_req_off": seg_req_off[:g + 1],
                "seg_tok_off": seg_tok_off[:g + 1], "n_segments": g}


def hmi_pool_prefetch(pool: int, layer: int, tenant_ids) -> int:
    ids = _i32(tenant_ids)
    return lib.hmi_pool_prefetch(pool, layer, _p32(ids), ids.shape[0])


def hmi_pool_stats(pool: int) -> dict:
    v = [C.c_int64(0) for _ in range(4)]
    lib.hmi_pool_stats(pool, *[C.byref(x) for x in v])
    return dict(zip(("hits", "misses", "bytes_h2d", "evictions"), (x.value for x in v)))


KERNEL_KINDS = ("router", "gemm", "attention", "layernorm")


def hmi_pool_profile(pool: int, enable: bool) -> int:
    return lib.hmi_pool_profile(pool, int(enable))


def hmi_pool_profile_read(pool: int):
    ms = (C.c_double * len(KERNEL_KINDS))()
    n = (C.c_int64 * len(KERNEL_KINDS))()
    rc = lib.hmi_pool_profile_read(pool, ms, n)
    return rc, {k: {"ms": ms[i], "launches": n[i]} for i, k in enumerate(KERNEL_KINDS)}


def hmi_pool_image_bytes(pool: int) -> int:
    return lib.hmi_pool_image_bytes(pool)


def hmi_pool_destroy(pool: Optional[int]) -> int:
    return lib.hmi_pool_destroy(pool)


def hmi_queue_create(pool: int, max_batch_requests: int, max_batch_tokens: int, max_waiting_batches: int):
    """-> (status, queue handle or None)."""
    out = C.c_void_p()
    rc = lib.hmi_queue_create(pool, max_batch_requests, max_batch_tokens, max_waiting_batches, C.byref(out))
    return rc, (out.value if rc == HMI_OK else None)


def hmi_queue_push(queue: int, tenant_id: int, seq_len: int, x_rows_ptr: int):
    """-> (status, ticket)."""
    t = C.c_int64(-1)
    rc = lib.hmi_queue_push(queue, tenant_id, seq_len, x_rows_ptr, C.byref(t))
    return rc, t.value


def hmi_queue_run(queue: int):
    """-> (status, batch number or -1, its number of requests)."""
    b, n = C.c_int64(-1), C.c_int32(0)
    rc = lib.hmi_queue_run(queue, C.byref(b), C.byref(n))
    return rc, b.value, n.value


def hmi_queue_fetch(queue: int, ticket: int, y_rows_ptr: int) -> int:
    return lib.hmi_queue_fetch(queue, ticket, y_rows_ptr)


def hmi_queue_waiting(queue: int) -> int:
    return lib.hmi_queue_waiting(queue)


def hmi_queue_last_error(queue: Optional[int]) -> str:
    return (lib.hmi_queue_last_error(queue) or b"").decode()


def hmi_queue_destroy(queue: Optional[int]) -> int:
    return lib.hmi_queue_destroy(queue)


# ---------------------------------------------------------------- convenience wrapper

class Pool:
    """Owns one hmi pool handle; raises HmiError on any non-zero status."""

    def __init__(self, **cfg):
        self.max_requests = cfg["max_requests"]
        rc, h = hmi_pool_create(**cfg)
        if rc != HMI_OK:
            raise HmiError(rc, hmi_last_error(None))
        self.h = h

    def _check(self, rc: int) -> None:
        if rc != HMI_OK:
            raise HmiError(rc, hmi_last_error(self.h))

    def load_tenant(self, tenant_id: int, layer: int, tensors) -> None:
        self._check(hmi_pool_load_tenant(self.h, tenant_id, layer, tensors))

    def alias_tenant(self, tenant_id: int, source_tenant: int) -> None:
        self._check(hmi_pool_alias_tenant(self.h, tenant_id, source_tenant))

    def load_shared(self, layer: int, tensors) -> None:
        self._check(hmi_pool_load_shared(self.h, layer, tensors))

    def plot_aggregate(self, table, frag_ids, seq_lens, x) -> None:
        """table [entries, 3, d] pool dtype, frag_ids int32 [N], x [N, d]: torch tensors on the device."""
        self._check(hmi_plot_aggregate(self.h, table.data_ptr(), table.shape[0], frag_ids.data_ptr(), seq_lens, x.data_ptr()))

    def kv_create(self, max_seqs: int, max_len: int) -> None:
        self._check(hmi_kv_create(self.h, max_seqs, max_len))

    def prefill(self, layer_begin: int, layer_end: int, x, y, tenant_ids, seq_lens, seq_slots) -> None:
        self._check(hmi_prefill(self.h, layer_begin, layer_end, x.data_ptr(), y.data_ptr(), tenant_ids, seq_lens, seq_slots))

    def decode_step(self, layer_begin: int, layer_end: int, x, y, tenant_ids, seq_slots) -> None:
        self._check(hmi_decode_step(self.h, layer_begin, layer_end, x.data_ptr(), y.data_ptr(), tenant_ids, seq_slots))

    def load_head(self, tenant_id: int, w, b, per_token: bool) -> None:
        self._check(hmi_pool_load_head(self.h, tenant_id, w, b, per_token))

    def head_forward(self, h, scores, labels) -> None:
        """h [N, d] pool dtype, scores float32 [N, max_classes] or None, labels int32 [N]: torch tensors on the device."""
        self._check(hmi_head_forward(self.h, h.data_ptr(), 0 if scores is None else scores.data_ptr(), labels.data_ptr()))

    def forward(self, layer: int, x, y, tenant_ids, seq_lens) -> None:
        """x, y: torch tensors on the pool's device ([N, d], pool dtype, contiguous)."""
        self._check(hmi_layer_forward(self.h, layer, x.data_ptr(), y.data_ptr(), tenant_ids, seq_lens))

    def forward_static(self, layer: int, x, y, tenant_ids, seq_lens) -> None:
        self._check(hmi_layer_forward_static(self.h, layer, x.data_ptr(), y.data_ptr(), tenant_ids, seq_lens))

    def stack_forward(self, layer_begin: int, layer_end: int, x, y, tenant_ids, seq_lens) -> None:
        self._check(hmi_stack_forward(self.h, layer_begin, layer_end, x.data_ptr(), y.data_ptr(),
                                      tenant_ids, seq_lens))

    def stack_forward_f32(self, layer_begin: int, layer_end: int, x, y, tenant_ids, seq_lens) -> None:
        """y: float32 tensor [N, d_model]; the last layer's result is not rounded to the storage type."""
        self._check(hmi_stack_forward_f32(self.h, layer_begin, layer_end, x.data_ptr(), y.data_ptr(),
                                          tenant_ids, seq_lens))

    def route(self) -> dict:
        rc, rt = hmi_get_route(self.h, self.max_requests)
        self._check(rc)
        return rt

    def prefetch(self, layer: int, tenant_ids) -> None:
        self._check(hmi_pool_prefetch(self.h, layer, tenant_ids))

    def profile(self, enable: bool) -> None:
        self._check(hmi_pool_profile(self.h, enable))

    def profile_read(self) -> dict:
        rc, out = hmi_pool_profile_read(self.h)
        self._check(rc)
        return out

    def stats(self) -> dict:
        return hmi_pool_stats(self.h)

    @property
    def image_bytes(self) -> int:
        return hmi_pool_image_bytes(self.h)

    def close(self) -> None:
        if self.h is not None:
            hmi_pool_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Queue:
    """Owns one request queue in front of a Pool; raises HmiError on any non-zero status except a full queue."""

    def __init__(self, pool: Pool, max_batch_requests: int, max_batch_tokens: int, max_waiting_batches: int = 2):
        self.pool = pool
        rc, h = hmi_queue_create(pool.h, max_batch_requests, max_batch_tokens, max_waiting_batches)
        if rc != HMI_OK:
            raise HmiError(rc, "hmi_queue_create failed")
        self.h = h

    def _check(self, rc: int) -> None:
        if rc != HMI_OK:
            raise HmiError(rc, hmi_queue_last_error(self.h))

    def push(self, tenant_id: int, x_rows):
        """x_rows: torch tensor [seq_len, d] on the device.  -> ticket, or None when the queue is full (run a batch first)."""
        rc, ticket = hmi_queue_push(self.h, tenant_id, x_rows.shape[0], x_rows.data_ptr())
        if rc == HMI_ERR_CAPACITY:
            return None
        self._check(rc)
        return ticket

    def run(self):
        """-> (batch number or -1, number of requests)."""
        rc, b, n = hmi_queue_run(self.h)
        self._check(rc)
        return b, n

    def fetch(self, ticket: int, y_rows) -> None:
        self._check(hmi_queue_fetch(self.h, ticket, y_rows.data_ptr()))

    def waiting(self) -> int:
        return hmi_queue_waiting(self.h)

    def close(self) -> None:
        if self.h is not None:
            hmi_queue_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
