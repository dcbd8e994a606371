"""ctypes binding of libkvprefetch.so: argument marshalling only.

Every step of the attention path runs in the library's HIP kernels; torch is used
for device memory and streams.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
import threading

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libkvprefetch.so")
_lib = None
_lock = threading.Lock()

KV_F16, KV_BF16, KV_I32, KV_F32 = 0, 1, 2, 3
KV_FP8_E4M3 = 4
_DTYPE_CODES = {torch.float16: KV_F16, torch.bfloat16: KV_BF16, torch.int32: KV_I32, torch.float32: KV_F32,
                torch.float8_e4m3fn: KV_FP8_E4M3}
KV_MAX_PREFETCH_DISTANCE = 4
KV_NOALLOC_SCRATCH_BYTES = 32 << 20


class KVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"kvprefetch status {status}: {message}")
        self.status = status


class KVTensor(ctypes.Structure):
    _fields_ = [
        ("data", ctypes.c_void_p),
        ("dtype", ctypes.c_int32),
        ("ndim", ctypes.c_int32),
        ("shape", ctypes.c_int64 * 5),
        ("stride", ctypes.c_int64 * 5),
    ]


EXPORTS = [
    "kv_decode_attn", "kv_decode_attn_noalloc", "kv_validate_inputs", "kv_decode_attn_kv8", "kv_decode_get_waves_per_cu_kv8", "kv_decode_layerstack", "kv_decode_workspace_bytes", "kv_layerstack_workspace_bytes",
    "kv_decode_set_workspace", "kv_decode_set_worker_trace", "kv_decode_set_xcd_skew", "kv_decode_fetch_probe",
    "kv_decode_set_l2_touch", "kv_decode_set_variant", "kv_decode_set_fetch_policy", "kv_decode_get_waves_per_cu_for",
    "kv_decode_set_waves_per_cu", "kv_decode_get_waves_per_cu", "kv_last_error", "kv_version",
    "kv_block_bytes", "kv_iter_working_set_bytes", "kv_worker_range", "kv_worker_of_tile", "kv_profile_enable", "kv_profile_read", "kv_profile_read_each",
]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libkvprefetch.so (built by ``build.build_library`` / ``__graft_entry__.build``)."""
    global _lib
    with _lock:
        if _lib is None:
            if not os.path.exists(_LIB_PATH):
                raise FileNotFoundError(
                    f"{_LIB_PATH} is not built; run `python -m paper_2504_06319_amd.build` first")
            lib = ctypes.CDLL(_LIB_PATH)
            T = ctypes.POINTER(KVTensor)
            TT = ctypes.POINTER(T)
            lib.kv_decode_attn.restype = ctypes.c_int
            lib.kv_decode_attn.argtypes = [T, T, T, T, T, T, ctypes.c_float, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_void_p]
            lib.kv_decode_attn_noalloc.restype = ctypes.c_int
            lib.kv_decode_attn_noalloc.argtypes = lib.kv_decode_attn.argtypes
            lib.kv_validate_inputs.restype = ctypes.c_int
            lib.kv_validate_inputs.argtypes = [T, T, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
            lib.kv_decode_fetch_probe.restype = ctypes.c_int
            lib.kv_decode_fetch_probe.argtypes = lib.kv_decode_attn.argtypes
            lib.kv_decode_attn_kv8.restype = ctypes.c_int
            lib.kv_decode_attn_kv8.argtypes = [T, T, T, T, T, T, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                               ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
            lib.kv_decode_layerstack.restype = ctypes.c_int
            lib.kv_decode_layerstack.argtypes = [ctypes.c_int, T, TT, T, TT, TT, TT, T, T, TT, ctypes.c_float,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_void_p]
            lib.kv_decode_workspace_bytes.restype = ctypes.c_size_t
            lib.kv_decode_workspace_bytes.argtypes = [ctypes.c_int] * 5
            lib.kv_layerstack_workspace_bytes.restype = ctypes.c_size_t
            lib.kv_layerstack_workspace_bytes.argtypes = [ctypes.c_int] * 3
            lib.kv_decode_set_workspace.restype = ctypes.c_int
            lib.kv_decode_set_workspace.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
            lib.kv_decode_set_worker_trace.restype = ctypes.c_int
            lib.kv_decode_set_worker_trace.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
            lib.kv_decode_set_waves_per_cu.restype = ctypes.c_int
            lib.kv_decode_set_waves_per_cu.argtypes = [ctypes.c_int]
            lib.kv_decode_get_waves_per_cu.restype = ctypes.c_int
            lib.kv_decode_get_waves_per_cu.argtypes = [ctypes.c_int, ctypes.c_int]
            lib.kv_profile_enable.restype = ctypes.c_int
            lib.kv_profile_enable.argtypes = [ctypes.c_int, ctypes.c_int]
            lib.kv_profile_read.restype = ctypes.c_int
            lib.kv_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
            lib.kv_profile_read_each.restype = ctypes.c_int
            lib.kv_profile_read_each.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
            lib.kv_last_error.restype = ctypes.c_char_p
            lib.kv_version.restype = ctypes.c_int
            lib.kv_worker_range.restype = ctypes.c_int
            lib.kv_worker_range.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
            lib.kv_worker_of_tile.restype = ctypes.c_int
            lib.kv_worker_of_tile.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int64]
            lib.kv_block_bytes.restype = ctypes.c_size_t
            lib.kv_block_bytes.argtypes = [ctypes.c_int] * 3
            lib.kv_iter_working_set_bytes.restype = ctypes.c_size_t
            lib.kv_iter_working_set_bytes.argtypes = [ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int]
            _lib = lib
    return _lib


def kv_last_error() -> str:
    return load_library().kv_last_error().decode()


def _check(status: int):
    if status != 0:
        raise KVError(status, kv_last_error())


def describe(t: torch.Tensor) -> KVTensor:
    """Descriptor of a torch tensor: pointer, dtype code, extents, element strides."""
    if t.dtype not in _DTYPE_CODES:
        raise KVError(1, f"unsupported torch dtype {t.dtype}")
    if t.dim() > 5:
        raise KVError(1, "tensors of rank > 5 are not supported")
    d = KVTensor()
    d.data = t.data_ptr()
    d.dtype = _DTYPE_CODES[t.dtype]
    d.ndim = t.dim()
    for i in range(t.dim()):
        d.shape[i] = t.shape[i]
        d.stride[i] = t.stride(i)
    return d


def _stream_handle(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


_workspaces: dict = {}
_registered: dict = {}          # device index -> (pointer, bytes) the library holds for that device


def _ensure_workspace(device: torch.device, nbytes: int):
    """Keep a torch-owned scratch buffer per device registered with the library (which keeps one per device and
    hands every calling stream its own slice): four times what one call can need, so that several streams fit."""
    lib = load_library()
    if nbytes == 0:
        return
    index = device.index if device.index is not None else torch.cuda.current_device()
    ws = _workspaces.get(index)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            torch.cuda.synchronize(index)        # registering again releases the slices earlier calls may still use
        ws = torch.empty(max(4 * nbytes, 1 << 20), dtype=torch.uint8, device=device)
        _workspaces[index] = ws
    if _registered.get(index) != (ws.data_ptr(), ws.numel()):
        with torch.cuda.device(index):
            _check(lib.kv_decode_set_workspace(ctypes.c_void_p(ws.data_ptr()), ws.numel()))
        _registered[index] = (ws.data_ptr(), ws.numel())


def _call(fn, device: torch.device):
    """Run a library call that takes a slice of the workspace.  When the workspace is used up by the slices of
    other streams (status 4), wait for the device, release every slice by registering the buffer again and try
    once more; not under a stream capture, where nothing may wait."""
    status = fn()
    index = device.index if device.index is not None else torch.cuda.current_device()
    ws = _workspaces.get(index)
    if status == 4 and ws is not None and not torch.cuda.is_current_stream_capturing():
        torch.cuda.synchronize(index)
        with torch.cuda.device(index):
            _check(load_library().kv_decode_set_workspace(ctypes.c_void_p(ws.data_ptr()), ws.numel()))
        status = fn()
    _check(status)


def kv_decode_workspace_bytes(B: int, Hq: int, d: int, max_context: int, block_size: int) -> int:
    return int(load_library().kv_decode_workspace_bytes(B, Hq, d, max_context, block_size))


def kv_layerstack_workspace_bytes(Hq: int, d: int, gemm_n: int) -> int:
    return int(load_library().kv_layerstack_workspace_bytes(Hq, d, gemm_n))


def kv_decode_set_worker_trace(buf):
    """Register an int64 device tensor of shape [workers, 4] for per-worker timestamps, or None to stop."""
    lib = load_library()
    if buf is None:
        _check(lib.kv_decode_set_worker_trace(None, 0))
        return
    if buf.dtype != torch.int64 or not buf.is_contiguous():
        raise KVError(1, "kv_decode_set_worker_trace: a contiguous int64 tensor is needed")
    _check(lib.kv_decode_set_worker_trace(ctypes.c_void_p(buf.data_ptr()), buf.numel() * 8))


def kv_decode_set_waves_per_cu(waves: int):
    _check(load_library().kv_decode_set_waves_per_cu(int(waves)))


def kv_decode_get_waves_per_cu(prefetch_distance: int, head_dim: int = 128) -> int:
    return int(load_library().kv_decode_get_waves_per_cu(int(prefetch_distance), int(head_dim)))


def kv_decode_attn(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                   block_size, prefetch_distance=1, stream=None):
    """Enqueue paged decode attention on ``stream`` (default: torch's current stream); returns ``out``."""
    lib = load_library()
    if q.dim() == 3 and block_tables.dim() == 2:
        need = kv_decode_workspace_bytes(q.shape[0], q.shape[1], q.shape[2],
                                         block_tables.shape[1] * block_size, block_size)
        _ensure_workspace(q.device, need)
    descs = [describe(t) for t in (q, k_cache, v_cache, block_tables, context_lens, out)]
    _call(lambda: lib.kv_decode_attn(*[ctypes.byref(d) for d in descs], float(scale), int(num_kv_heads),
                                     int(block_size), int(prefetch_distance), ctypes.c_void_p(_stream_handle(stream))), q.device)
    return out


def kv_decode_attn_noalloc(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                           block_size, prefetch_distance=1, stream=None):
    """kv_decode_attn on the library's static scratch array: no workspace is created or registered here, and
    nothing on this path allocates device memory."""
    lib = load_library()
    descs = [describe(t) for t in (q, k_cache, v_cache, block_tables, context_lens, out)]
    _check(lib.kv_decode_attn_noalloc(*[ctypes.byref(d) for d in descs], float(scale), int(num_kv_heads),
                                      int(block_size), int(prefetch_distance), ctypes.c_void_p(_stream_handle(stream))))
    return out


def kv_validate_inputs(block_tables, context_lens, num_blocks, block_size, stream=None):
    """Synchronising check of the lengths and of every block id in use; raises KVError naming the first bad entry."""
    dbt, dcl = describe(block_tables), describe(context_lens)
    _check(load_library().kv_validate_inputs(ctypes.byref(dbt), ctypes.byref(dcl), int(num_blocks), int(block_size),
                                             ctypes.c_void_p(_stream_handle(stream))))


def kv_decode_fetch_probe(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                          block_size, prefetch_distance=1, stream=None):
    """The fetch stream of kv_decode_attn without its arithmetic (a measurement aid); writes nothing."""
    lib = load_library()
    need = kv_decode_workspace_bytes(q.shape[0], q.shape[1], q.shape[2],
                                     block_tables.shape[1] * block_size, block_size)
    _ensure_workspace(q.device, need)
    descs = [describe(t) for t in (q, k_cache, v_cache, block_tables, context_lens, out)]
    _call(lambda: lib.kv_decode_fetch_probe(*[ctypes.byref(d) for d in descs], float(scale), int(num_kv_heads), int(block_size),
                                            int(prefetch_distance), ctypes.c_void_p(_stream_handle(stream))), q.device)


def kv_decode_attn_kv8(q, k_cache, v_cache, block_tables, context_lens, out, scale, k_scale, v_scale,
                       num_kv_heads, block_size, prefetch_distance=1, stream=None):
    """Paged decode attention over an FP8 E4M3 cache (torch.float8_e4m3fn, or uint8 codes)."""
    lib = load_library()
    need = kv_decode_workspace_bytes(q.shape[0], q.shape[1], q.shape[2],
                                     block_tables.shape[1] * block_size, block_size)
    if need:
        _ensure_workspace(q.device, need)
    caches = [c.view(torch.float8_e4m3fn) if c.dtype == torch.uint8 else c for c in (k_cache, v_cache)]
    descs = [describe(t) for t in (q, caches[0], caches[1], block_tables, context_lens, out)]
    _call(lambda: lib.kv_decode_attn_kv8(*[ctypes.byref(d) for d in descs], float(scale), float(k_scale), float(v_scale),
                                         int(num_kv_heads), int(block_size), int(prefetch_distance),
                                         ctypes.c_void_p(_stream_handle(stream))), q.device)
    return out


KV_VARIANT_ONE_PASS, KV_VARIANT_TWO_PHASE = 0, 1
KV_FETCH_NON_TEMPORAL, KV_FETCH_PLAIN = 0, 1
KV_PREFETCH_AUTO = -1


def kv_decode_set_fetch_policy(policy: int):
    _check(load_library().kv_decode_set_fetch_policy(int(policy)))


def kv_decode_set_variant(variant: int):
    _check(load_library().kv_decode_set_variant(int(variant)))


def kv_decode_set_l2_touch(tiles: int):
    _check(load_library().kv_decode_set_l2_touch(int(tiles)))


def kv_decode_set_xcd_skew(per_1024: int):
    _check(load_library().kv_decode_set_xcd_skew(int(per_1024)))


def kv_decode_get_waves_per_cu_for(prefetch_distance: int, head_dim: int, q_heads_per_kv_head: int) -> int:
    return int(load_library().kv_decode_get_waves_per_cu_for(int(prefetch_distance), int(head_dim), int(q_heads_per_kv_head)))


def kv_decode_get_waves_per_cu_kv8(prefetch_distance: int, head_dim: int = 128) -> int:
    return int(load_library().kv_decode_get_waves_per_cu_kv8(int(prefetch_distance), int(head_dim)))


def _desc_array(tensors):
    descs = [describe(t) for t in tensors]
    arr = (ctypes.POINTER(KVTensor) * len(descs))(*[ctypes.pointer(d) for d in descs])
    return arr, descs


def kv_decode_layerstack(x, weights, gemm_out, q, k_caches, v_caches, block_tables, context_lens, outs,
                         scale, num_kv_heads, block_size, prefetch_distance=1, cross_layer_prefetch=0,
                         stream=None):
    """Enqueue the GEMM + attention layer stack; ``q`` may be None (queries come from the GEMM output)."""
    lib = load_library()
    L = len(weights)
    o0 = outs[0]
    need = kv_decode_workspace_bytes(o0.shape[0], o0.shape[1], o0.shape[2],
                                     block_tables.shape[1] * block_size, block_size)
    if any(w.dim() == 5 for w in weights):
        need = max(need, kv_layerstack_workspace_bytes(o0.shape[1], o0.shape[2], gemm_out.shape[1]))
    _ensure_workspace(x.device, need)
    w_arr, w_keep = _desc_array(weights)
    k_arr, k_keep = _desc_array(k_caches)
    v_arr, v_keep = _desc_array(v_caches)
    o_arr, o_keep = _desc_array(outs)
    if q is not None:
        q_arr, q_keep = _desc_array(q)
    else:
        q_arr, q_keep = None, None
    dx, dg, dbt, dcl = describe(x), describe(gemm_out), describe(block_tables), describe(context_lens)
    _call(lambda: lib.kv_decode_layerstack(L, ctypes.byref(dx), w_arr, ctypes.byref(dg), q_arr, k_arr, v_arr,
                                           ctypes.byref(dbt), ctypes.byref(dcl), o_arr, float(scale),
                                           int(num_kv_heads), int(block_size), int(prefetch_distance),
                                           int(cross_layer_prefetch), ctypes.c_void_p(_stream_handle(stream))), x.device)
    return outs


def kv_profile_enable(max_calls: int, every: int = 1):
    _check(load_library().kv_profile_enable(int(max_calls), int(every)))


def kv_profile_read():
    """(main kernel ms summed, calls) since the last read."""
    a, n = ctypes.c_double(), ctypes.c_int()
    _check(load_library().kv_profile_read(ctypes.byref(a), ctypes.byref(n)))
    return a.value, n.value


def kv_profile_read_each(capacity: int = 100000):
    """Main-kernel milliseconds of every sampled call since the last read, as a list."""
    buf, n = (ctypes.c_float * capacity)(), ctypes.c_int()
    _check(load_library().kv_profile_read_each(buf, capacity, ctypes.byref(n)))
    return list(buf[: n.value])


def pack_weights(w: torch.Tensor, layout: str = "operand") -> torch.Tensor:
    """Re-lay a [K, N] weight matrix for the dense layer; set-up time, pure data movement.

    ``"operand"``: [N/64, K/32, 4, 64, 8], the order in which the matrix cores read the B operand,
    ``Wp[t, ks, nb, l, j] = W[32 ks + 8 (l // 16) + j, 64 t + 16 nb + l % 16]`` (K must be 1024, 2048, 4096 or
    8192): the fast path, weights go from HBM straight into registers.
    ``"tile"``: [N/128, K, 128], one contiguous run per 128-column tile, for the kernel that stages W through LDS.
    """
    K, N = w.shape
    if layout == "tile":
        if N % 128:
            raise KVError(1, "pack_weights: N must be a multiple of 128")
        return w.reshape(K, N // 128, 128).permute(1, 0, 2).contiguous()
    if layout != "operand":
        raise KVError(1, f"pack_weights: unknown layout {layout!r}")
    if N % 64 or K % 32:
        raise KVError(1, "pack_weights: N must be a multiple of 64 and K of 32")
    # W[ks, lq, j, t, nb, lr] -> Wp[t, ks, nb, (lq, lr), j]
    return (w.reshape(K // 32, 4, 8, N // 64, 4, 16).permute(3, 0, 4, 1, 5, 2).contiguous()
            .reshape(N // 64, K // 32, 4, 64, 8))


def kv_worker_range(tiles: int, workers: int, xcd_skew: int, worker: int):
    first, end = ctypes.c_int64(), ctypes.c_int64()
    _check(load_library().kv_worker_range(tiles, workers, xcd_skew, worker, ctypes.byref(first), ctypes.byref(end)))
    return first.value, end.value


def kv_worker_of_tile(tiles: int, workers: int, xcd_skew: int, tile: int) -> int:
    return int(load_library().kv_worker_of_tile(tiles, workers, xcd_skew, tile))


def kv_block_bytes(elem_bytes: int, head_dim: int, block_size: int) -> int:
    return int(load_library().kv_block_bytes(elem_bytes, head_dim, block_size))


def kv_iter_working_set_bytes(block_bytes: int, units_per_wg: int, H: int, B: int) -> int:
    return int(load_library().kv_iter_working_set_bytes(block_bytes, units_per_wg, H, B))


def kv_version() -> int:
    return int(load_library().kv_version())
