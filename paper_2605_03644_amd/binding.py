"""Thin ctypes binding of libadapshot (include/adapshot.h).

Argument marshalling only: every step of the hot path runs in the library's HIP
kernels.  torch is used for device memory (`tensor.data_ptr()`) and for the
current stream.  There is no fallback: if the shared library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ADAPSHOT_LIB", os.path.join(_HERE, "libadapshot.so"))

OK, EINVAL, ESHOT, ECAPACITY, ESTATE, EDEVICE = range(6)
STATUS_NAMES = {OK: "OK", EINVAL: "EINVAL", ESHOT: "ESHOT", ECAPACITY: "ECAPACITY", ESTATE: "ESTATE",
                EDEVICE: "EDEVICE"}
F32, BF16 = 0, 1
KEYS_UNROTATED, KEYS_ROTATED_LOCAL = 0, 1

# every symbol declared in include/adapshot.h
EXPORTS = ["adapshot_create", "adapshot_destroy", "adapshot_last_error", "adapshot_version",
           "adapshot_pool_register", "adapshot_assemble", "adapshot_query_attn", "adapshot_probe_entropy",
           "adapshot_profile_enable", "adapshot_profile_read", "adapshot_profile_read_each", "adapshot_assemble_batched",
           "adapshot_query_attn_batched", "adapshot_decode_append", "adapshot_probe_entropy_tokens",
           "adapshot_pick_shots", "adapshot_rank_shots", "adapshot_top_k", "adapshot_set_attn_splits",
           "adapshot_probe_entropy_static", "adapshot_query_attn_pool", "adapshot_query_attn_pool_batched",
           "adapshot_attn_split_plan"]
ENTROPY_FULL_P, ENTROPY_RENORMALISED = 0, 1
KERNEL_KINDS = ["assemble_reencode", "rope_rows", "query_attn", "attn_combine", "entropy_chunk", "entropy_finish"]


class ModelDesc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("rope_theta", ctypes.c_double), ("dtype", ctypes.c_int32),
                ("key_state", ctypes.c_int32), ("max_position", ctypes.c_int64)]


class CacheStruct(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("capacity", ctypes.c_int64),
                ("len", ctypes.c_int64), ("slot_shot", ctypes.c_void_p), ("slot_tok", ctypes.c_void_p),
                ("slot_pos", ctypes.c_void_p)]


class AttnItem(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("k_self", ctypes.c_void_p), ("v_self", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("n_ctx", ctypes.c_int64), ("q_pos0", ctypes.c_int64),
                ("t_q", ctypes.c_int32), ("cache_index", ctypes.c_int32)]


class AdapshotError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"adapshot {STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libadapshot.so (built in-tree by paper_2605_03644_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2605_03644_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.adapshot_create.restype = ctypes.c_int
    L.adapshot_create.argtypes = [ctypes.POINTER(ModelDesc), ctypes.POINTER(vp)]
    L.adapshot_destroy.restype = None
    L.adapshot_destroy.argtypes = [vp]
    L.adapshot_last_error.restype = ctypes.c_char_p
    L.adapshot_last_error.argtypes = [vp]
    L.adapshot_version.restype = ctypes.c_char_p
    L.adapshot_version.argtypes = []
    L.adapshot_pool_register.restype = ctypes.c_int
    L.adapshot_pool_register.argtypes = [vp, vp, vp, vp, i32, i64]
    L.adapshot_assemble.restype = ctypes.c_int
    L.adapshot_assemble.argtypes = [vp, ctypes.POINTER(CacheStruct), vp, vp, i32, i64, vp]
    L.adapshot_query_attn.restype = ctypes.c_int
    L.adapshot_query_attn.argtypes = [vp, ctypes.POINTER(CacheStruct), i32, i64, vp, vp, vp, i32, i64, vp, vp]
    L.adapshot_query_attn_pool.restype = ctypes.c_int
    L.adapshot_query_attn_pool.argtypes = [vp, i32, vp, vp, i32, i64, vp, vp, vp, i32, i64, vp, vp]
    L.adapshot_probe_entropy.restype = ctypes.c_int
    L.adapshot_probe_entropy.argtypes = [vp, vp, i64, i32, i32, vp, vp]
    L.adapshot_probe_entropy_static.restype = ctypes.c_int
    L.adapshot_probe_entropy_static.argtypes = [vp, vp, i64, i32, i32, vp, vp]
    L.adapshot_probe_entropy_tokens.restype = ctypes.c_int
    L.adapshot_probe_entropy_tokens.argtypes = [vp, vp, i64, i32, i32, vp, i32, i32, vp, vp]
    L.adapshot_rank_shots.restype = ctypes.c_int
    L.adapshot_rank_shots.argtypes = [vp, i32, vp, i32, i64, vp, vp]
    L.adapshot_top_k.restype = ctypes.c_int
    L.adapshot_top_k.argtypes = [vp, vp, i32, i32, vp]
    L.adapshot_pick_shots.restype = ctypes.c_int
    L.adapshot_pick_shots.argtypes = [vp, vp, vp, i32, ctypes.c_float, vp]
    L.adapshot_assemble_batched.restype = ctypes.c_int
    L.adapshot_assemble_batched.argtypes = [vp, ctypes.POINTER(CacheStruct), i32, vp, vp, vp, i64, vp]
    L.adapshot_query_attn_pool_batched.restype = ctypes.c_int
    L.adapshot_query_attn_pool_batched.argtypes = [vp, i32, vp, vp, vp, i32, i64, ctypes.POINTER(AttnItem), i32, vp]
    L.adapshot_query_attn_batched.restype = ctypes.c_int
    L.adapshot_query_attn_batched.argtypes = [vp, ctypes.POINTER(CacheStruct), i32, i32, ctypes.POINTER(AttnItem), i32, vp]
    L.adapshot_decode_append.restype = ctypes.c_int
    L.adapshot_decode_append.argtypes = [vp, ctypes.POINTER(CacheStruct), i32, vp, vp, i64, vp]
    L.adapshot_attn_split_plan.restype = ctypes.c_int
    L.adapshot_attn_split_plan.argtypes = [ctypes.POINTER(ModelDesc), i32, i32, i64, ctypes.POINTER(i32), ctypes.POINTER(i64)]
    L.adapshot_set_attn_splits.restype = ctypes.c_int
    L.adapshot_set_attn_splits.argtypes = [vp, i32]
    L.adapshot_profile_enable.restype = ctypes.c_int
    L.adapshot_profile_enable.argtypes = [vp, i32]
    L.adapshot_profile_read.restype = ctypes.c_int
    L.adapshot_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.adapshot_profile_read_each.restype = ctypes.c_int
    L.adapshot_profile_read_each.argtypes = [vp, i32, vp, i64, ctypes.POINTER(i64)]
    _lib = L
    return L


def attn_split_plan(n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, n_compute_units: int, t_q: int,
                    n_ctx: int):
    """(n_split, keys_per_split) of one adapshot_query_attn call (host logic only: runs without a GPU)."""
    desc = ModelDesc(1, n_q_heads, n_kv_heads, head_dim, 1.0e4, dtype, KEYS_UNROTATED, 0)
    ns, kps = ctypes.c_int32(), ctypes.c_int64()
    st = load_library().adapshot_attn_split_plan(ctypes.byref(desc), n_compute_units, t_q, n_ctx, ctypes.byref(ns),
                                                 ctypes.byref(kps))
    if st != OK:
        raise AdapshotError(st, "attn_split_plan: bad arguments")
    return ns.value, kps.value


def _stream_ptr(stream: Optional[torch.cuda.Stream] = None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _torch_dtype(dtype: int) -> torch.dtype:
    return torch.float32 if dtype == F32 else torch.bfloat16


class Cache:
    """Caller-owned assembled cache: k, v [L, capacity, H_kv, d] plus optional per-slot index arrays."""

    def __init__(self, ctx: "Context", capacity: int, with_index: bool = True, device=None):
        d = ctx.desc
        dev = device if device is not None else ctx.device
        shape = (d.n_layers, capacity, d.n_kv_heads, d.head_dim)
        self.k = torch.zeros(shape, dtype=_torch_dtype(d.dtype), device=dev)
        self.v = torch.zeros(shape, dtype=_torch_dtype(d.dtype), device=dev)
        self.slot_shot = torch.full((capacity,), -1, dtype=torch.int32, device=dev) if with_index else None
        self.slot_tok = torch.full((capacity,), -1, dtype=torch.int32, device=dev) if with_index else None
        self.slot_pos = torch.full((capacity,), -1, dtype=torch.int64, device=dev) if with_index else None
        self.c = CacheStruct(self.k.data_ptr(), self.v.data_ptr(), capacity, 0,
                             self.slot_shot.data_ptr() if with_index else None,
                             self.slot_tok.data_ptr() if with_index else None,
                             self.slot_pos.data_ptr() if with_index else None)

    @property
    def len(self) -> int:
        return int(self.c.len)

    @property
    def capacity(self) -> int:
        return int(self.c.capacity)

    def reset(self) -> None:
        self.c.len = 0


class Context:
    """One model shape on the current device (adapshot_create / adapshot_destroy)."""

    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_theta: float,
                 dtype: int, key_state: int = KEYS_UNROTATED, max_position: int = 0):
        self.lib = load_library()
        self.desc = ModelDesc(n_layers, n_q_heads, n_kv_heads, head_dim, float(rope_theta), dtype, key_state,
                              max_position)
        self._h = ctypes.c_void_p()
        self.n_shots = 0  # set by pool_register
        st = self.lib.adapshot_create(ctypes.byref(self.desc), ctypes.byref(self._h))
        if st != OK:
            raise AdapshotError(st, "adapshot_create failed (bad model description or no usable HIP device)")
        self.device = torch.device("cuda", torch.cuda.current_device())
        self._keep = []

    @classmethod
    def for_workload(cls, w, key_state: int = KEYS_UNROTATED, n_layers: Optional[int] = None,
                     max_position: int = 0) -> "Context":
        return cls(w.n_layers if n_layers is None else n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim,
                   w.rope_theta, F32 if w.dtype == "f32" else BF16, key_state, max_position)

    def close(self) -> None:
        if self._h:
            self.lib.adapshot_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self.lib.adapshot_last_error(self._h).decode()

    def _check(self, st: int) -> None:
        if st != OK:
            raise AdapshotError(st, self.last_error())

    # -- adapshot_pool_register
    def pool_register(self, k_pool: torch.Tensor, v_pool: torch.Tensor, shot_offsets: np.ndarray) -> None:
        off = np.ascontiguousarray(shot_offsets, dtype=np.int64)
        assert k_pool.is_contiguous() and v_pool.is_contiguous() and k_pool.shape == v_pool.shape
        self._check(self.lib.adapshot_pool_register(self._h, k_pool.data_ptr(), v_pool.data_ptr(),
                                                    off.ctypes.data, off.shape[0] - 1, k_pool.shape[1]))
        self._keep = [k_pool, v_pool]  # the library borrows the pool: keep it alive, and only once it is accepted
        self.n_shots = int(off.shape[0] - 1)

    # -- adapshot_assemble
    def assemble(self, cache: Cache, shot_ids: Sequence[int], order: Optional[Sequence[int]] = None,
                 pos0: int = 0, stream: Optional[torch.cuda.Stream] = None) -> None:
        ids = np.ascontiguousarray(shot_ids, dtype=np.int32)
        od = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
        self._check(self.lib.adapshot_assemble(self._h, ctypes.byref(cache.c), ids.ctypes.data,
                                               None if od is None else od.ctypes.data, ids.shape[0], pos0,
                                               _stream_ptr(stream)))

    # -- adapshot_query_attn
    def query_attn(self, cache: Cache, layer: int, n_ctx: int, q: torch.Tensor, k_self: torch.Tensor,
                   v_self: torch.Tensor, q_pos0: int, out: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert q.is_contiguous() and k_self.is_contiguous() and v_self.is_contiguous()
        if out is None:
            out = torch.empty_like(q)
        self._check(self.lib.adapshot_query_attn(self._h, ctypes.byref(cache.c), layer, n_ctx, q.data_ptr(),
                                                 k_self.data_ptr(), v_self.data_ptr(), q.shape[0], q_pos0,
                                                 out.data_ptr(), _stream_ptr(stream)))
        return out

    # -- adapshot_query_attn_pool (zero-copy form)
    def query_attn_pool(self, layer: int, shot_ids: Sequence[int], order: Optional[Sequence[int]], q: torch.Tensor,
                        k_self: torch.Tensor, v_self: torch.Tensor, q_pos0: int, pos0: int = 0,
                        out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert q.is_contiguous() and k_self.is_contiguous() and v_self.is_contiguous()
        ids = np.ascontiguousarray(shot_ids, dtype=np.int32)
        od = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
        if out is None:
            out = torch.empty_like(q)
        self._check(self.lib.adapshot_query_attn_pool(self._h, layer, ids.ctypes.data,
                                                      None if od is None else od.ctypes.data, ids.shape[0], pos0,
                                                      q.data_ptr(), k_self.data_ptr(), v_self.data_ptr(), q.shape[0],
                                                      q_pos0, out.data_ptr(), _stream_ptr(stream)))
        return out

    # -- adapshot_probe_entropy
    def probe_entropy(self, logits: torch.Tensor, out: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
        rows, vocab = logits.shape
        if out is None:
            out = torch.empty(rows, dtype=torch.float32, device=logits.device)
        self._check(self.lib.adapshot_probe_entropy(self._h, logits.data_ptr(), logits.stride(0) if rows > 1 else vocab,
                                                    rows, vocab, out.data_ptr(), _stream_ptr(stream)))
        return out

    # -- adapshot_probe_entropy_static: `out` is required (the call itself allocates nothing)
    def probe_entropy_static(self, logits: torch.Tensor, out: torch.Tensor,
                             stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
        rows, vocab = logits.shape
        assert out.dtype == torch.float32 and out.numel() >= rows
        self._check(self.lib.adapshot_probe_entropy_static(self._h, logits.data_ptr(),
                                                           logits.stride(0) if rows > 1 else vocab, rows, vocab,
                                                           out.data_ptr(), _stream_ptr(stream)))
        return out

    # -- adapshot_probe_entropy_tokens
    def probe_entropy_tokens(self, logits: torch.Tensor, token_ids, mode: int = ENTROPY_FULL_P,
                             out: Optional[torch.Tensor] = None,
                             stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
        rows, vocab = logits.shape
        ids = np.ascontiguousarray(np.asarray(token_ids, dtype=np.int32))
        if out is None:
            out = torch.empty(rows, dtype=torch.float32, device=logits.device)
        self._check(self.lib.adapshot_probe_entropy_tokens(
            self._h, logits.data_ptr(), logits.stride(0) if rows > 1 else vocab, rows, vocab,
            ids.ctypes.data_as(ctypes.c_void_p), int(ids.size), int(mode), out.data_ptr(), _stream_ptr(stream)))
        return out

    # -- adapshot_rank_shots / adapshot_top_k
    def rank_shots(self, layer: int, q: torch.Tensor, q_pos0: int = 0, out: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert q.is_contiguous() and q.dim() == 3
        if out is None:
            out = torch.empty(self.n_shots, dtype=torch.float32, device=q.device)
        self._check(self.lib.adapshot_rank_shots(self._h, int(layer), q.data_ptr(), int(q.shape[0]), int(q_pos0),
                                                 out.data_ptr(), _stream_ptr(stream)))
        return out

    def top_k(self, scores, k: int) -> np.ndarray:
        sc = np.ascontiguousarray(np.asarray(scores, dtype=np.float32))
        ids = np.empty(int(k), np.int32)
        self._check(self.lib.adapshot_top_k(self._h, sc.ctypes.data_as(ctypes.c_void_p), int(sc.size), int(k),
                                            ids.ctypes.data_as(ctypes.c_void_p)))
        return ids

    # -- adapshot_pick_shots (host logic)
    def pick_shots(self, entropy, shot_counts, tau: float) -> int:
        h = np.ascontiguousarray(np.asarray(entropy, dtype=np.float32))
        k = np.ascontiguousarray(np.asarray(shot_counts, dtype=np.int32))
        assert h.shape == k.shape and h.ndim == 1
        picked = ctypes.c_int32(0)
        self._check(self.lib.adapshot_pick_shots(self._h, h.ctypes.data_as(ctypes.c_void_p),
                                                 k.ctypes.data_as(ctypes.c_void_p), int(h.size), float(tau),
                                                 ctypes.byref(picked)))
        return int(picked.value)

    # -- batched forms: the C structs of several caches are packed into one array for the call and the
    #    advanced lengths are copied back
    @staticmethod
    def _pack_caches(caches):
        arr = (CacheStruct * len(caches))()
        for i, c in enumerate(caches):
            arr[i] = c.c
        return arr

    @staticmethod
    def _unpack_lens(caches, arr):
        for i, c in enumerate(caches):
            c.c.len = arr[i].len

    # -- adapshot_assemble_batched
    def assemble_batched(self, caches, shot_ids, orders=None, pos0: int = 0,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
        n = len(caches)
        ids = [np.ascontiguousarray(x, dtype=np.int32) for x in shot_ids]
        ods = None if orders is None else [None if o is None else np.ascontiguousarray(o, dtype=np.int32) for o in orders]
        id_ptrs = (ctypes.c_void_p * n)(*[x.ctypes.data for x in ids])
        od_ptrs = None if ods is None else (ctypes.c_void_p * n)(*[None if o is None else o.ctypes.data for o in ods])
        m = np.array([x.shape[0] for x in ids], dtype=np.int32)
        arr = self._pack_caches(caches)
        st = self.lib.adapshot_assemble_batched(self._h, arr, n, ctypes.cast(id_ptrs, ctypes.c_void_p),
                                                None if od_ptrs is None else ctypes.cast(od_ptrs, ctypes.c_void_p),
                                                m.ctypes.data, pos0, _stream_ptr(stream))
        self._unpack_lens(caches, arr)
        self._check(st)

    # -- adapshot_query_attn_batched: items = [(cache_index, n_ctx, q, k_self, v_self, q_pos0, out)]
    @staticmethod
    def pack_attn_items(items):
        """The C array of a list of (cache_index, n_ctx, q, k_self, v_self, q_pos0, out); reusable across calls
        as long as the tensors stay alive and the lengths do not change."""
        its = (AttnItem * len(items))()
        for i, (ci, n_ctx, q, ks, vs, q_pos0, out) in enumerate(items):
            assert q.is_contiguous() and ks.is_contiguous() and vs.is_contiguous() and out.is_contiguous()
            its[i] = AttnItem(q.data_ptr(), ks.data_ptr(), vs.data_ptr(), out.data_ptr(), n_ctx, q_pos0, q.shape[0], ci)
        return its

    def query_attn_batched(self, caches, layer: int, items, stream: Optional[torch.cuda.Stream] = None) -> None:
        """items: a list of (cache_index, n_ctx, q, k_self, v_self, q_pos0, out), or what pack_attn_items made of one."""
        arr = self._pack_caches(caches)
        its = items if isinstance(items, ctypes.Array) else self.pack_attn_items(items)
        self._check(self.lib.adapshot_query_attn_batched(self._h, arr, len(caches), layer, its, len(its),
                                                         _stream_ptr(stream)))

    # -- adapshot_query_attn_pool_batched (zero-copy form): an item's cache_index names a shot list
    def pack_shot_lists(self, shot_ids, orders=None):
        """The C arrays of n shot lists (and their orders); reusable across calls (one per layer)."""
        n = len(shot_ids)
        ids = [np.ascontiguousarray(x, dtype=np.int32) for x in shot_ids]
        ods = None if orders is None else [None if o is None else np.ascontiguousarray(o, dtype=np.int32) for o in orders]
        id_ptrs = (ctypes.c_void_p * n)(*[x.ctypes.data for x in ids])
        od_ptrs = None if ods is None else (ctypes.c_void_p * n)(*[None if o is None else o.ctypes.data for o in ods])
        m = np.array([x.shape[0] for x in ids], dtype=np.int32)
        return (ids, ods, id_ptrs, od_ptrs, m)

    def query_attn_pool_batched(self, layer: int, lists, items, pos0: int = 0,
                                stream: Optional[torch.cuda.Stream] = None) -> None:
        """lists: what pack_shot_lists returned, or (shot_ids, orders); items as in query_attn_batched with the list
        index in place of the cache index."""
        if len(lists) == 2:
            lists = self.pack_shot_lists(lists[0], lists[1])
        _, _, id_ptrs, od_ptrs, m = lists
        its = items if isinstance(items, ctypes.Array) else self.pack_attn_items(items)
        self._check(self.lib.adapshot_query_attn_pool_batched(
            self._h, layer, ctypes.cast(id_ptrs, ctypes.c_void_p),
            None if od_ptrs is None else ctypes.cast(od_ptrs, ctypes.c_void_p), m.ctypes.data, m.shape[0], pos0,
            its, len(its), _stream_ptr(stream)))

    # -- adapshot_decode_append: k_new, v_new [L, n_caches, H_kv, d]
    def decode_append(self, caches, k_new: torch.Tensor, v_new: torch.Tensor, pos0: int = 0,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
        assert k_new.shape[1] == len(caches)
        arr = self._pack_caches(caches)
        st = self.lib.adapshot_decode_append(self._h, arr, len(caches), k_new.data_ptr(), v_new.data_ptr(), pos0,
                                             _stream_ptr(stream))
        self._unpack_lens(caches, arr)
        self._check(st)

    # -- adapshot_set_attn_splits
    def set_attn_splits(self, n_split: int) -> None:
        self._check(self.lib.adapshot_set_attn_splits(self._h, int(n_split)))

    # -- adapshot_profile_enable / adapshot_profile_read
    def profile_enable(self, on: bool) -> None:
        self._check(self.lib.adapshot_profile_enable(self._h, 1 if on else 0))

    def profile_read(self) -> dict:
        """{kernel kind: (total_ms, launches)} of the launches recorded since the last read."""
        out = {}
        for kind, name in enumerate(KERNEL_KINDS):
            ms, n = ctypes.c_double(), ctypes.c_int64()
            self._check(self.lib.adapshot_profile_read(self._h, kind, ctypes.byref(ms), ctypes.byref(n)))
            out[name] = (ms.value, n.value)
        return out

    def profile_read_each(self, capacity: int = 1 << 16) -> dict:
        """{kernel kind: float32 array of the durations in ms, in launch order} of the launches recorded since
        the last read (at most `capacity` per kind are returned)."""
        out = {}
        for kind, name in enumerate(KERNEL_KINDS):
            buf = np.empty(capacity, np.float32)
            n = ctypes.c_int64()
            self._check(self.lib.adapshot_profile_read_each(self._h, kind, buf.ctypes.data_as(ctypes.c_void_p),
                                                            capacity, ctypes.byref(n)))
            out[name] = buf[:min(n.value, capacity)].copy()
        return out
