"""ctypes front end of the plain CPU oracle (oracle/adapshot_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU-baseline
leg may import this package; the product package never does, and this package
never imports the product.  `build()` compiles the C file with gcc; every call
below is argument marshalling around one C function.

Array conventions: fp32 tensors are numpy float32, bf16 tensors are numpy uint16
bit patterns; `dtype` is "f32" or "bf16".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# ADAPSHOT_ORACLE_SRC points the loader at another copy of the C file (the mutation check of the pins
# compiles deliberately broken copies in a scratch directory); the library is built next to it.
_SRC = os.environ.get("ADAPSHOT_ORACLE_SRC", os.path.join(_HERE, "adapshot_oracle.c"))
_LIB = os.path.join(os.path.dirname(os.path.abspath(_SRC)), "libadapshot_oracle.so")

F32, BF16 = 0, 1
KEYS_UNROTATED, KEYS_ROTATED_LOCAL = 0, 1
_DT = {"f32": F32, "bf16": BF16}
_NP = {"f32": np.float32, "bf16": np.uint16}

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle (gcc -O2, OpenMP across independent units, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        i32, i64, f64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        L.adapshot_oracle_threads.restype = i32
        L.adapshot_oracle_double_to_bf16.restype = ctypes.c_uint16
        L.adapshot_oracle_double_to_bf16.argtypes = [f64]
        L.adapshot_oracle_plan.restype = i64
        L.adapshot_oracle_plan.argtypes = [vp, i32, vp, vp, i32, i64, i64, vp, vp, vp, vp]
        L.adapshot_oracle_rot.restype = None
        L.adapshot_oracle_rot.argtypes = [vp, i32, f64, f64, vp]
        L.adapshot_oracle_rot_rows.restype = None
        L.adapshot_oracle_rot_rows.argtypes = [vp, ctypes.c_int, i64, i32, f64, vp, vp, vp]
        L.adapshot_oracle_assemble.restype = ctypes.c_int
        L.adapshot_oracle_assemble.argtypes = [vp, vp, ctypes.c_int, i32, i64, i32, i32, f64, ctypes.c_int,
                                               vp, vp, vp, i64, i64, vp, vp, i64, vp]
        L.adapshot_oracle_query_attn.restype = ctypes.c_int
        L.adapshot_oracle_query_attn.argtypes = [vp, vp, ctypes.c_int, i64, vp, vp, vp, i32, i32, i32, i32,
                                                 f64, i64, vp, i64, vp]
        L.adapshot_oracle_entropy.restype = None
        L.adapshot_oracle_entropy.argtypes = [vp, i64, i32, i32, vp]
        L.adapshot_oracle_entropy_subset.restype = None
        L.adapshot_oracle_entropy_subset.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp]
        L.adapshot_oracle_rank_scores.restype = ctypes.c_int
        L.adapshot_oracle_rank_scores.argtypes = [vp, ctypes.c_int, vp, i32, vp, i32, i32, i32, i32, f64,
                                                  ctypes.c_int, i64, vp]
        L.adapshot_oracle_pick_shots.restype = i32
        L.adapshot_oracle_pick_shots.argtypes = [vp, vp, i32, f64]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def threads() -> int:
    return int(lib().adapshot_oracle_threads())


def double_to_bf16(x: float) -> int:
    return int(lib().adapshot_oracle_double_to_bf16(float(x)))


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def plan(shot_offsets, shot_ids, order, slot0: int = 0, pos0: int = 0):
    """-> dict(n, slot_shot, slot_tok, slot_pos, slot_src); raises ValueError on a bad id."""
    so = _chk(np.asarray(shot_offsets), np.int64)
    ids = _chk(np.asarray(shot_ids, dtype=np.int32), np.int32)
    od = None if order is None else _chk(np.asarray(order, dtype=np.int32), np.int32)
    m = int(ids.shape[0])
    n = lib().adapshot_oracle_plan(_p(so), so.shape[0] - 1, _p(ids), _p(od), m, slot0, pos0,
                                   None, None, None, None)
    if n < 0:
        raise ValueError("shot id or order entry out of range")
    out = dict(n=int(n), slot_shot=np.empty(n, np.int32), slot_tok=np.empty(n, np.int32),
               slot_pos=np.empty(n, np.int64), slot_src=np.empty(n, np.int64))
    lib().adapshot_oracle_plan(_p(so), so.shape[0] - 1, _p(ids), _p(od), m, slot0, pos0,
                               _p(out["slot_shot"]), _p(out["slot_tok"]), _p(out["slot_pos"]), _p(out["slot_src"]))
    return out


def rot(x: np.ndarray, base: float, a: float) -> np.ndarray:
    x = _chk(np.asarray(x, dtype=np.float64), np.float64)
    y = np.empty_like(x)
    lib().adapshot_oracle_rot(_p(x), x.shape[-1], float(base), float(a), _p(y))
    return y


def rot_rows(x: np.ndarray, dtype: str, base: float, angles, want_exact: bool = False):
    """x: [..., d] in storage type; angles: one angle multiplier per row.  Returns rows rotated and
    rounded to the storage type (and the fp64 rows before rounding if want_exact)."""
    x = _chk(x, _NP[dtype])
    d = x.shape[-1]
    n = x.size // d
    a = _chk(np.ascontiguousarray(angles, dtype=np.float64).reshape(-1), np.float64)
    if a.shape[0] != n:
        raise ValueError("one angle per row expected")
    y = np.empty_like(x)
    ex = np.empty(x.shape, np.float64) if want_exact else None
    lib().adapshot_oracle_rot_rows(_p(x), _DT[dtype], n, d, float(base), _p(a), _p(y), _p(ex))
    return (y, ex) if want_exact else y


def assemble(k_pool: np.ndarray, v_pool: np.ndarray, dtype: str, base: float, key_state: int,
             pl: dict, slot0: int, capacity: int, k_out: Optional[np.ndarray] = None,
             v_out: Optional[np.ndarray] = None, want_exact: bool = False):
    """k_pool, v_pool: [L, pool_tokens, H_kv, d] in storage type.  Returns (k_out, v_out, k_exact|None)
    with k_out, v_out [L, capacity, H_kv, d] (slots outside the appended range untouched/zero)."""
    k_pool = _chk(k_pool, _NP[dtype]); v_pool = _chk(v_pool, _NP[dtype])
    L, ptok, hkv, d = k_pool.shape
    if k_out is None:
        k_out = np.zeros((L, capacity, hkv, d), _NP[dtype])
    if v_out is None:
        v_out = np.zeros((L, capacity, hkv, d), _NP[dtype])
    n = pl["n"]
    k_exact = np.empty((L, n, hkv, d), np.float64) if want_exact else None
    rc = lib().adapshot_oracle_assemble(_p(k_pool), _p(v_pool), _DT[dtype], L, ptok, hkv, d, float(base),
                                        int(key_state), _p(pl["slot_src"]), _p(pl["slot_tok"]),
                                        _p(pl["slot_pos"]), n, slot0, _p(k_out), _p(v_out), capacity, _p(k_exact))
    if rc != 0:
        raise ValueError("oracle assemble: bad arguments (capacity or head_dim)")
    return k_out, v_out, k_exact


def query_attn(k_cache: np.ndarray, v_cache: np.ndarray, dtype: str, n_ctx: int, q: np.ndarray,
               k_self: np.ndarray, v_self: np.ndarray, base: float, q_pos0: int,
               pairs: Optional[np.ndarray] = None) -> np.ndarray:
    """k_cache, v_cache: one layer [>=n_ctx, H_kv, d]; q [T_q, H_q, d]; k_self, v_self [T_q, H_kv, d].
    Returns fp64 [T_q, H_q, d], or [n_pairs, d] for the given (row j, head h) pairs."""
    st = _NP[dtype]
    k_cache = _chk(k_cache, st); v_cache = _chk(v_cache, st)
    q = _chk(q, st); k_self = _chk(k_self, st); v_self = _chk(v_self, st)
    t_q, h_q, d = q.shape
    h_kv = k_self.shape[1]
    if k_cache.shape[0] < n_ctx:
        raise ValueError("n_ctx exceeds the cache rows given")
    if pairs is None:
        out = np.empty((t_q, h_q, d), np.float64)
        npairs = 0
    else:
        pairs = _chk(np.asarray(pairs, dtype=np.int32), np.int32)
        npairs = pairs.shape[0]
        out = np.empty((npairs, d), np.float64)
    rc = lib().adapshot_oracle_query_attn(_p(k_cache), _p(v_cache), _DT[dtype], n_ctx, _p(q), _p(k_self),
                                          _p(v_self), t_q, h_q, h_kv, d, float(base), q_pos0,
                                          _p(pairs), npairs, _p(out))
    if rc != 0:
        raise ValueError("oracle query_attn: bad arguments")
    return out


def entropy(logits: np.ndarray) -> np.ndarray:
    """logits fp32 [rows, V] (last dim contiguous) -> fp64 [rows], natural log."""
    if logits.dtype != np.float32 or logits.ndim != 2 or logits.strides[1] != 4:
        raise TypeError("logits must be float32 [rows, vocab] with a contiguous vocab axis")
    rows, vocab = logits.shape
    out = np.empty(rows, np.float64)
    lib().adapshot_oracle_entropy(_p(logits), logits.strides[0] // 4, rows, vocab, _p(out))
    return out


ENTROPY_FULL_P, ENTROPY_RENORMALISED = 0, 1


def entropy_subset(logits: np.ndarray, ids, mode: int) -> np.ndarray:
    """Eq. (entropy) summed over the answer tokens `ids` only; mode ENTROPY_FULL_P or ENTROPY_RENORMALISED."""
    if logits.dtype != np.float32 or logits.ndim != 2 or logits.strides[1] != 4:
        raise TypeError("logits must be float32 [rows, vocab] with a contiguous vocab axis")
    rows, vocab = logits.shape
    ids = _chk(np.asarray(ids, dtype=np.int32), np.int32)
    if ids.ndim != 1 or len(set(ids.tolist())) != ids.size or ids.min() < 0 or ids.max() >= vocab:
        raise ValueError("ids must be distinct token indices inside the vocabulary")
    out = np.empty(rows, np.float64)
    lib().adapshot_oracle_entropy_subset(_p(logits), logits.strides[0] // 4, rows, vocab, _p(ids), ids.size, int(mode), _p(out))
    return out


def pick_shots(h, counts, tau: float) -> int:
    """Smallest candidate count whose probe entropy is <= tau, or -1."""
    h = _chk(np.asarray(h, dtype=np.float64), np.float64)
    counts = _chk(np.asarray(counts, dtype=np.int32), np.int32)
    if h.shape != counts.shape or h.ndim != 1:
        raise ValueError("h and counts must be 1-D of equal length")
    return int(lib().adapshot_oracle_pick_shots(_p(h), _p(counts), h.size, float(tau)))


def rank_scores(k_pool: np.ndarray, dtype: str, shot_offsets, q: np.ndarray, base: float, key_state: int,
                q_pos0: int = 0) -> np.ndarray:
    """Relevance s^(i) of every shot (Eq. attention_score, softmax over the whole pool).
    k_pool: one layer [tokens, H_kv, d]; q [T_q, H_q, d]; returns fp64 [n_shots]."""
    st = _NP[dtype]
    k_pool = _chk(k_pool, st); q = _chk(q, st)
    off = _chk(np.asarray(shot_offsets, dtype=np.int64), np.int64)
    t_q, h_q, d = q.shape
    h_kv = k_pool.shape[1]
    if k_pool.shape[0] < off[-1] or k_pool.shape[2] != d:
        raise ValueError("pool layer smaller than the shot offsets say")
    out = np.empty(off.size - 1, np.float64)
    rc = lib().adapshot_oracle_rank_scores(_p(k_pool), _DT[dtype], _p(off), off.size - 1, _p(q), t_q, h_q, h_kv, d,
                                           float(base), int(key_state), int(q_pos0), _p(out))
    if rc != 0:
        raise ValueError("oracle rank_scores: bad arguments")
    return out
