"""ctypes binding of libexpertweave.so: argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels; PyTorch supplies device
memory and the current stream.  There is no fallback: if the library is missing or a call
fails, an exception is raised.  Function names mirror include/expertweave.h.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libexpertweave.so")

EW_F32, EW_BF16 = 0, 1
EW_POOL_VMM, EW_POOL_PADDED, EW_POOL_FAKE, EW_POOL_EAGER_UNMAP = 0, 1, 2, 4
ERR_NAMES = {0: "EW_OK", -1: "EW_ERR_INVALID_ARG", -2: "EW_ERR_OOM", -3: "EW_ERR_VMM", -4: "EW_ERR_STATE",
             -5: "EW_ERR_WORKSPACE", -6: "EW_ERR_UNSUPPORTED", -7: "EW_ERR_HIP"}

# name -> (restype, argtypes); mirrors include/expertweave.h
_i32p, _f32p, _vp, _sz, _int = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p, C.c_size_t, C.c_int
SIGNATURES = {
    "ew_last_error": (C.c_char_p, []),
    "ew_abi_version": (_int, []),
    "expert_pool_create": (_int, [C.POINTER(_vp), _int, _int, _int, _int, _int, _sz, _sz, _sz, _sz, _int]),
    "expert_pool_destroy": (_int, [_vp]),
    "expert_pool_map": (_int, [_vp, _int, _int, _int, _vp, _vp, _vp, _vp]),
    "expert_pool_unmap": (_int, [_vp, _int, _int, _vp]),
    "expert_pool_view": (_int, [_vp, _int, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_int)]),
    "expert_pool_expert_map_host": (_int, [_vp, _int, _vp]),
    "expert_pool_touch": (_int, [_vp, _int, _vp]),
    "expert_pool_lru_victim": (_int, [_vp, C.POINTER(C.c_int)]),
    "expert_pool_stats": (_int, [_vp, _vp]),
    "expert_pool_trim": (_int, [_vp, _sz]),
    "expert_pool_fake_fail_at": (_int, [_vp, _int, _int]),
    "expert_pool_fake_is_mapped": (_int, [_vp, _int, _int, _sz, C.POINTER(_int)]),
    "moe_route_topk": (_int, [_vp, _int, _int, _int, _int, _vp, _vp, _vp]),
    "moe_reroute_permute_workspace_bytes": (_sz, [_int, _int, _int]),
    "moe_reroute_permute": (_int, [_vp, _vp, _vp, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_reroute_permute_static_max_bytes": (_sz, []),
    "moe_reroute_permute_static": (_int, [_vp, _vp, _vp, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_route_reroute_permute": (_int, [_vp, _vp, _vp, _int, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp,
                                         _vp, _vp, _vp, _sz, _vp]),
    "moe_route_reroute_permute_plan": (_int, [_vp, _vp, _vp, _int, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp,
                                              _vp, _vp, _vp, _sz, _int, _int, _int, _int, _vp, _sz, _vp]),
    "moe_reroute_singleop_workspace_bytes": (_sz, [_int, _int]),
    "moe_reroute_singleop": (_int, [_vp, _vp, _vp, _int, _int, _int, _int, _vp, _vp, _sz, _vp]),
    "moe_grouped_ffn_workspace_bytes": (_sz, [_int, _int, _int, _int, _int, _int]),
    "moe_grouped_ffn": (_int, [_vp, _int, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_grouped_ffn_planned": (_int, [_vp, _int, _int, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                       _vp, _vp, _sz, _vp]),
    "moe_grouped_ffn_with_shared": (_int, [_vp, _int, _int, _int, _int, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                           _vp, _vp, _sz, _vp]),
    "moe_unpermute": (_int, [_vp, _vp, _vp, _vp, _int, _vp, _int, _int, _int, _int, _vp, _vp]),
    "moe_unpermute_rmsnorm": (_int, [_vp, _vp, _vp, _vp, _int, _vp, _int, _int, _int, _int, _vp, C.c_float, _vp, _vp]),
    "moe_gate_logits": (_int, [_vp, _int, _vp, _int, _int, _int, _vp, _vp, _vp, _vp]),
    "moe_rmsnorm": (_int, [_vp, _int, _int, _int, C.c_float, _vp, _vp]),
    "ew_probe_stream": (_int, [_vp, _vp, _sz, _int, _vp]),
    "ew_probe_mfma_bf16": (_int, [_int, _int, _int, _vp, _vp]),
    "ew_tune_ffn": (None, [_int, _int, _int, _int, _int, _int, _int]),
    "ew_tune_route": (None, [_int]),
}


class PoolStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("page_bytes", "bytes_virtual", "pages_mapped", "pages_free", "pages_parked", "pages_created",
                                          "pages_released", "pages_shared", "bytes_experts", "experts_loaded")] + \
               [("f_mem", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class EWError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2508_17624_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2508_17624_amd.build`; "
                               "there is no fallback path")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(rc: int):
    if rc != 0:
        raise EWError(rc, lib().ew_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return EW_F32
    if t.dtype == torch.bfloat16:
        return EW_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _workspace(nbytes: int, device) -> torch.Tensor | None:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device) if nbytes else None


# ----------------------------------------------------------------------------- expert pool
class ExpertPool:
    """Owns an ew_pool*.  Weights handed to map() may be CPU or CUDA tensors (or None)."""

    def __init__(self, num_layers, M, N, E_max, w13_bytes, w2_bytes, page_bytes=0, prealloc_pages=0,
                 flags=EW_POOL_VMM, device=0):
        self._h = C.c_void_p()
        _check(lib().expert_pool_create(C.byref(self._h), device, num_layers, M, N, E_max, w13_bytes, w2_bytes,
                                        page_bytes, prealloc_pages, flags))
        self.L, self.M, self.N, self.E_max, self.P = num_layers, M, N, E_max, M + N * E_max
        self.flags, self.device = flags, device
        self._keep = []

    @property
    def fake(self):
        return bool(self.flags & EW_POOL_FAKE)

    def close(self):
        if self._h:
            _check(lib().expert_pool_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def map(self, layer, adapter_id, expert_ids, w13=None, w2=None, stream=None):
        ids = None
        n = 0
        if expert_ids is not None:
            ids = (C.c_int32 * len(expert_ids))(*[int(e) for e in expert_ids])
            n = len(expert_ids)
        for w in (w13, w2):
            if w is not None and not w.is_contiguous():
                raise ValueError("weights must be contiguous")
        st = stream if stream is not None else (None if self.fake else _stream())
        _check(lib().expert_pool_map(self._h, layer, adapter_id, n, C.cast(ids, C.c_void_p) if ids is not None else None,
                                     _ptr(w13), _ptr(w2), st))
        if not self.fake:
            torch.cuda.current_stream().synchronize()      # host sources may be freed by the caller afterwards

    def unmap(self, layer, adapter_id):
        _check(lib().expert_pool_unmap(self._h, layer, adapter_id, None if self.fake else _stream()))

    def view(self, layer):
        """(w13_base, w2_base, expert_map_ptr, P) as integers."""
        a, b, m, p = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_int()
        _check(lib().expert_pool_view(self._h, layer, C.byref(a), C.byref(b), C.byref(m), C.byref(p)))
        return a.value, b.value, m.value, p.value

    def expert_map_host(self, layer):
        out = torch.empty((self.N + 1, self.M), dtype=torch.int32)
        _check(lib().expert_pool_expert_map_host(self._h, layer, out.data_ptr()))
        return out

    def touch(self, adapter_ids):
        """Marks the adapters of a scheduled batch as just used (eviction order)."""
        ids = (C.c_int32 * len(adapter_ids))(*[int(a) for a in adapter_ids])
        _check(lib().expert_pool_touch(self._h, len(adapter_ids), ids))

    def lru_victim(self) -> int:
        """The loaded adapter used least recently, or -1."""
        out = C.c_int(-1)
        _check(lib().expert_pool_lru_victim(self._h, C.byref(out)))
        return out.value

    def stats(self) -> dict:
        s = PoolStats()
        _check(lib().expert_pool_stats(self._h, C.byref(s)))
        return s.as_dict()

    def trim(self, keep_pages=0):
        _check(lib().expert_pool_trim(self._h, keep_pages))

    def fake_fail_at(self, op, n):
        _check(lib().expert_pool_fake_fail_at(self._h, op, n))

    def fake_is_mapped(self, layer, which, offset) -> bool:
        out = C.c_int()
        _check(lib().expert_pool_fake_is_mapped(self._h, layer, which, offset, C.byref(out)))
        return bool(out.value)


# ----------------------------------------------------------------------------- hot path
def moe_route_topk(logits: torch.Tensor, k: int, renormalize: bool = False):
    T, E = logits.shape
    ids = torch.empty((T, k), dtype=torch.int32, device=logits.device)
    w = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    _check(lib().moe_route_topk(_ptr(logits), T, E, k, int(renormalize), _ptr(ids), _ptr(w), _stream()))
    return ids, w


def moe_reroute_permute(topk_ids, adapter_id, expert_map, N: int, P: int, E: int | None = None, want_row_of_pair=True,
                        ws=None):
    """expert_map: int32 tensor [N+1, E] on the device, or a raw device pointer (then pass E)."""
    T, k = topk_ids.shape
    if E is None:
        E = expert_map.shape[1]
    dev = topk_ids.device
    slot = torch.empty((T, k), dtype=torch.int32, device=dev)
    counts = torch.empty(P, dtype=torch.int32, device=dev)
    offsets = torch.empty(P + 1, dtype=torch.int32, device=dev)
    por = torch.empty(T * k, dtype=torch.int32, device=dev)
    rop = torch.empty(T * k, dtype=torch.int32, device=dev) if want_row_of_pair else None
    need = lib().moe_reroute_permute_workspace_bytes(T, k, P)
    ws = ws if ws is not None else _workspace(need, dev)
    _check(lib().moe_reroute_permute(_ptr(topk_ids), _ptr(adapter_id), _ptr(expert_map), T, k, E, N, P, _ptr(slot),
                                     _ptr(counts), _ptr(offsets), _ptr(por), _ptr(rop), _ptr(ws),
                                     ws.numel() if ws is not None else 0, _stream()))
    return slot, counts, offsets, por, rop


def moe_reroute_permute_static(topk_ids, adapter_id, expert_map, N: int, P: int, out, E: int | None = None):
    """The variant that allocates nothing: `out` = (slot [T,k], counts [P], offsets [P+1], pair_of_row [T*k],
    row_of_pair [T*k] or None), all preallocated by the caller; scratch is the library's built-in buffer."""
    T, k = topk_ids.shape
    if E is None:
        E = expert_map.shape[1]
    slot, counts, offsets, por, rop = out
    _check(lib().moe_reroute_permute_static(_ptr(topk_ids), _ptr(adapter_id), _ptr(expert_map), T, k, E, N, P, _ptr(slot),
                                            _ptr(counts), _ptr(offsets), _ptr(por), _ptr(rop), _stream()))
    return out


def moe_route_reroute_permute(logits, adapter_id, expert_map, k: int, N: int, P: int, renormalize=False, ws=None):
    T, E = logits.shape
    dev = logits.device
    ids = torch.empty((T, k), dtype=torch.int32, device=dev)
    w = torch.empty((T, k), dtype=torch.float32, device=dev)
    slot = torch.empty((T, k), dtype=torch.int32, device=dev)
    counts = torch.empty(P, dtype=torch.int32, device=dev)
    offsets = torch.empty(P + 1, dtype=torch.int32, device=dev)
    por = torch.empty(T * k, dtype=torch.int32, device=dev)
    rop = torch.empty(T * k, dtype=torch.int32, device=dev)
    need = lib().moe_reroute_permute_workspace_bytes(T, k, P)
    ws = ws if ws is not None else _workspace(need, dev)
    _check(lib().moe_route_reroute_permute(_ptr(logits), _ptr(adapter_id), _ptr(expert_map), T, E, k, N, P,
                                           int(renormalize), _ptr(ids), _ptr(w), _ptr(slot), _ptr(counts), _ptr(offsets),
                                           _ptr(por), _ptr(rop), _ptr(ws), ws.numel() if ws is not None else 0,
                                           _stream()))
    return ids, w, slot, counts, offsets, por, rop


def moe_reroute_singleop(topk_ids, adapter_id, expert_map, N: int, ws=None, out=None):
    """The unfused rerouting baseline (three launches); returns slot_ids [T, k]."""
    T, k = topk_ids.shape
    E = expert_map.shape[1]
    slot = out if out is not None else torch.empty((T, k), dtype=torch.int32, device=topk_ids.device)
    ws = ws if ws is not None else _workspace(lib().moe_reroute_singleop_workspace_bytes(T, k), topk_ids.device)
    _check(lib().moe_reroute_singleop(_ptr(topk_ids), _ptr(adapter_id), _ptr(expert_map), T, k, E, N, _ptr(slot), _ptr(ws),
                                      ws.numel() if ws is not None else 0, _stream()))
    return slot


def moe_grouped_ffn(x, k: int, I: int, P: int, counts, offsets, pair_of_row, w13_base, w2_base, ws=None, out=None,
                    num_rows: int | None = None):
    """w13_base / w2_base: device tensors [P, 2I, H] / [P, H, I] or raw device pointers (pool views).
    num_rows = offsets[P], the number of sorted rows; defaults to x.shape[0] * k.  It differs from
    that only when rows do not come from a top-k (shared experts: num_rows = S * T with k = 1)."""
    H = x.shape[1]
    rows = x.shape[0] * k if num_rows is None else num_rows
    if rows % k:
        raise ValueError("num_rows must be a multiple of k")
    T = rows // k
    dt = _dtype_code(x)
    y = out if out is not None else torch.empty((rows, H), dtype=x.dtype, device=x.device)
    if y.shape[0] < rows:
        raise ValueError("output has fewer rows than num_rows")
    need = lib().moe_grouped_ffn_workspace_bytes(T, k, H, I, P, dt)
    ws = ws if ws is not None else _workspace(need, x.device)
    _check(lib().moe_grouped_ffn(_ptr(x), dt, T, k, H, I, P, _ptr(counts), _ptr(offsets), _ptr(pair_of_row),
                                 _ptr(w13_base), _ptr(w2_base), _ptr(y), _ptr(ws), ws.numel() if ws is not None else 0,
                                 _stream()))
    return y


def moe_grouped_ffn_with_shared(x, k: int, I: int, P: int, counts, offsets, pair_of_row, w13_base, w2_base, w13_shared,
                                w2_shared, ws=None, out=None):
    """Routed and shared experts in one call.  w13_shared / w2_shared: [S, 2I, H] / [S, H, I].  Returns y [T*(k+S), H]:
    the routed rows, then the shared experts' [S, T, H] outputs (y[T*k:] is moe_unpermute's shared_out)."""
    T, H = x.shape
    S = w13_shared.shape[0]
    dt = _dtype_code(x)
    rows = T * (k + S)
    y = out if out is not None else torch.empty((rows, H), dtype=x.dtype, device=x.device)
    if y.shape[0] < rows:
        raise ValueError("output has fewer than T*(k+S) rows")
    need = lib().moe_grouped_ffn_workspace_bytes(T, k + S, H, I, P + S, dt)
    ws = ws if ws is not None else _workspace(need, x.device)
    _check(lib().moe_grouped_ffn_with_shared(_ptr(x), dt, T, k, H, I, P, S, _ptr(counts), _ptr(offsets), _ptr(pair_of_row),
                                             _ptr(w13_base), _ptr(w2_base), _ptr(w13_shared), _ptr(w2_shared), _ptr(y),
                                             _ptr(ws), ws.numel() if ws is not None else 0, _stream()))
    return y


def moe_unpermute(y_sorted, row_of_pair, topk_w, shared_out=None, out=None, residual=None):
    """shared_out: [S, T, H] (or [S*T, H]) slabs of shared-expert outputs, or None; residual: [T, H] or None."""
    T, k = topk_w.shape
    H = y_sorted.shape[1]
    S = 0 if shared_out is None else shared_out.numel() // (T * H)
    o = out if out is not None else torch.empty((T, H), dtype=y_sorted.dtype, device=y_sorted.device)
    _check(lib().moe_unpermute(_ptr(y_sorted), _ptr(row_of_pair), _ptr(topk_w), _ptr(shared_out), S, _ptr(residual), T, k, H,
                               _dtype_code(y_sorted), _ptr(o), _stream()))
    return o


def moe_unpermute_rmsnorm(y_sorted, row_of_pair, topk_w, eps: float, shared_out=None, out=None, normed_out=None, residual=None):
    """moe_unpermute and moe_rmsnorm of its result in one launch; returns (out, normed_out)."""
    T, k = topk_w.shape
    H = y_sorted.shape[1]
    S = 0 if shared_out is None else shared_out.numel() // (T * H)
    o = out if out is not None else torch.empty((T, H), dtype=y_sorted.dtype, device=y_sorted.device)
    n = normed_out if normed_out is not None else torch.empty_like(o)
    _check(lib().moe_unpermute_rmsnorm(_ptr(y_sorted), _ptr(row_of_pair), _ptr(topk_w), _ptr(shared_out), S, _ptr(residual), T, k,
                                       H, _dtype_code(y_sorted), _ptr(o), eps, _ptr(n), _stream()))
    return o, n


def tune_ffn(path: int = 0, stream_token_tiles: int = 0, stream_threads: int = 0, ws_frags: int = 0,
             ws_chunk_frags: int = 0, ws_wait_ticks: int = -1, ws_two_launches: bool = False):
    """Kernel-selection override of moe_grouped_ffn(bf16), process-global; no arguments = automatic.
    path 1 = register-streaming kernel (stream_token_tiles 1|2, stream_threads), 2 = LDS-tiled GEMM kernel,
    3 = LDS-direct streaming kernel (ws_frags 1|2|4|8 = kernel shape, ws_chunk_frags = cap on 32-row fragments
    per row chunk, ws_wait_ticks = rendezvous wait in 10 ns ticks, 0 = never, negative = automatic,
    ws_two_launches = decode shapes run their two products as two launches instead of one)."""
    lib().ew_tune_ffn(path, stream_token_tiles, stream_threads, ws_frags, ws_chunk_frags, ws_wait_ticks, int(ws_two_launches))


def tune_route(small_pairs: int = 2048):
    """Pairs (T*k) up to which moe_reroute_permute / moe_route_reroute_permute take the single-block permutation (with the router fused: a multi-block top-k kernel, then that block)."""
    lib().ew_tune_route(small_pairs)


def moe_gate_logits(x, Wg, adapter_id=None, bias=None):
    T, H = x.shape
    E = Wg.shape[0]
    logits = torch.empty((T, E), dtype=torch.float32, device=x.device)
    _check(lib().moe_gate_logits(_ptr(x), _dtype_code(x), _ptr(Wg), T, H, E, _ptr(adapter_id), _ptr(bias), _ptr(logits),
                                 _stream()))
    return logits


def moe_rmsnorm(x, eps: float = 1e-6, out=None):
    T, H = x.shape
    o = out if out is not None else torch.empty_like(x)
    _check(lib().moe_rmsnorm(_ptr(x), _dtype_code(x), T, H, float(eps), _ptr(o), _stream()))
    return o
