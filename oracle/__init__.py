"""CPU oracle for the Prompt Cache hot path -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes face over ``pc_oracle.c`` (plain fp64 C written from the
paper) plus ``toy.py`` (a tiny fp64 transformer used to pin the paper's
"cached modules == full pass under a module-local mask" equivalence).

Nothing here is imported by the product package; nothing here imports it.
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pc_oracle.c")
_LIB = os.path.join(_HERE, "libpc_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile pc_oracle.c with the host C compiler (no GPU toolchain involved)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _bind(path: str):
    """Open a build of pc_oracle.c and declare its functions' signatures."""
    lib = ctypes.CDLL(path)
    c_int, c_long, c_dbl, c_sz = ctypes.c_int, ctypes.c_long, ctypes.c_double, ctypes.c_size_t
    P = ctypes.c_void_p
    lib.orc_set_threads.argtypes = [c_int]
    lib.orc_set_threads.restype = c_int
    lib.orc_layout.argtypes = [c_int, P, P, P]
    lib.orc_layout.restype = c_long
    lib.orc_text_positions.argtypes = [c_int, c_int, c_int, P]
    lib.orc_text_positions.restype = None
    lib.orc_rope.argtypes = [P, c_int, c_int, c_int, P, c_dbl]
    lib.orc_rope.restype = None
    lib.orc_assemble.argtypes = [c_int, P, P, P, P, c_sz, P, P, P]
    lib.orc_assemble.restype = c_long
    lib.orc_attn.argtypes = [P, P, c_int, P, P, P, c_int, c_int, c_int, c_int, c_dbl, P]
    lib.orc_attn.restype = None
    lib.orc_alibi_slopes.argtypes = [c_int, P]
    lib.orc_alibi_slopes.restype = None
    lib.orc_attn_alibi.argtypes = [P, P, c_int, P, P, P, c_int, c_int, c_int, c_int, P, P]
    lib.orc_attn_alibi.restype = None
    lib.orc_full_masked.argtypes = [P, P, P, P, P, c_int, c_int, c_int, c_int, c_dbl, P, P]
    lib.orc_full_masked.restype = None
    lib.orc_fill_param.argtypes = [P, P, P, c_int, c_int, P, P, c_int, c_int, c_int, c_dbl]
    lib.orc_fill_param.restype = c_int
    lib.orc_bytes_per_token.argtypes = [c_int, c_int, c_int, c_int]
    lib.orc_bytes_per_token.restype = c_long
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(_LIB)
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def set_threads(n: int) -> int:
    return int(_load().orc_set_threads(int(n)))


# ----------------------------------------------------------------- layout
def layout(sizes: Sequence[int], union_ids: Sequence[int] | None = None):
    """Start position of each schema entry and the schema's total span (Sec. 3.3)."""
    n = len(sizes)
    size = np.ascontiguousarray(np.asarray(sizes, dtype=np.intc))
    uid = np.ascontiguousarray(
        np.full(n, -1, dtype=np.intc) if union_ids is None else np.asarray(union_ids, dtype=np.intc))
    start = np.zeros(n, dtype=np.intc)
    span = _load().orc_layout(n, _ptr(size), _ptr(uid), _ptr(start))
    if span < 0:
        raise ValueError("invalid schema: negative size or non-adjacent union children")
    return [int(s) for s in start], int(span)


def text_positions(prev_start: int, prev_len: int, n_tokens: int) -> np.ndarray:
    """Position IDs of uncached text placed right after an imported module (Sec. 3.4)."""
    pos = np.zeros(n_tokens, dtype=np.int32)
    _load().orc_text_positions(int(prev_start), int(prev_len), int(n_tokens), _ptr(pos))
    return pos


# ------------------------------------------------------------------- rope
def rope(x, pos, base: float = 10000.0) -> np.ndarray:
    """RoPE of x[tokens, heads, d] at arbitrary integer positions; returns a new fp64 array."""
    y = _f64(x).copy()
    assert y.ndim == 3 and y.shape[2] % 2 == 0
    p = _i32(pos)
    assert p.shape == (y.shape[0],)
    _load().orc_rope(_ptr(y), y.shape[0], y.shape[1], y.shape[2], _ptr(p), float(base))
    return y


# --------------------------------------------------------------- assemble
def assemble(mod_K: Sequence[np.ndarray], mod_V: Sequence[np.ndarray], mod_start: Sequence[int]):
    """Packed concatenation of module K/V rows (any dtype, copied as bytes) + position IDs.

    mod_K[m], mod_V[m]: arrays [len_m, ...] of identical trailing shape and dtype.
    Returns (out_K, out_V, out_pos) with out_K/out_V of that dtype and out_pos int32.
    """
    n = len(mod_K)
    assert n == len(mod_V) == len(mod_start)
    if n == 0:
        return None, None, np.zeros(0, dtype=np.int32)
    ks = [np.ascontiguousarray(k) for k in mod_K]
    vs = [np.ascontiguousarray(v) for v in mod_V]
    trailing, dtype = ks[0].shape[1:], ks[0].dtype
    row_bytes = int(np.prod(trailing)) * dtype.itemsize
    for k, v in zip(ks, vs):
        assert k.shape[1:] == trailing and v.shape == k.shape and k.dtype == dtype == v.dtype
    lens = np.asarray([k.shape[0] for k in ks], dtype=np.intc)
    starts = np.ascontiguousarray(np.asarray(mod_start, dtype=np.intc))
    total = int(lens.sum())
    out_K = np.zeros((total,) + trailing, dtype=dtype)
    out_V = np.zeros((total,) + trailing, dtype=dtype)
    out_pos = np.zeros(total, dtype=np.int32)
    PP = ctypes.c_void_p * n
    kp = PP(*[k.ctypes.data for k in ks])
    vp = PP(*[v.ctypes.data for v in vs])
    rows = _load().orc_assemble(n, ctypes.cast(kp, ctypes.c_void_p), ctypes.cast(vp, ctypes.c_void_p),
                                _ptr(lens), _ptr(starts), row_bytes, _ptr(out_K), _ptr(out_V), _ptr(out_pos))
    assert rows == total
    return out_K, out_V, out_pos


# -------------------------------------------------------------- attention
def attn(Q, q_pos, K, V, k_pos, base: float = 10000.0) -> np.ndarray:
    """Uncached-token attention over assembled KV (Sec. 3.4).

    Q [nq,Hq,d] raw (rotated inside at q_pos); K [nkv,Hkv,d] already encoded; V [nkv,Hkv,d].
    Key j is visible to query q iff k_pos[j] <= q_pos[q].  Returns fp64 [nq,Hq,d].
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    qp, kp = _i32(q_pos), _i32(k_pos)
    nq, Hq, d = Q.shape
    nkv, Hkv, d2 = K.shape
    assert d == d2 and V.shape == K.shape and Hq % Hkv == 0
    assert qp.shape == (nq,) and kp.shape == (nkv,)
    out = np.zeros((nq, Hq, d), dtype=np.float64)
    _load().orc_attn(_ptr(Q), _ptr(qp), nq, _ptr(K), _ptr(V), _ptr(kp), nkv, Hq, Hkv, d, float(base), _ptr(out))
    return out


def alibi_slopes(n_heads: int) -> np.ndarray:
    """Per-head slopes of the linear attention bias (Sec. 4.2, ALiBi): 8 heads -> 1/2 ... 1/256."""
    out = np.zeros(n_heads, dtype=np.float64)
    _load().orc_alibi_slopes(int(n_heads), _ptr(out))
    return out


def attn_alibi(Q, q_pos, K, V, k_pos, slopes) -> np.ndarray:
    """Uncached-token attention with the linear bias -slope[h] * (q_pos - k_pos) on position IDs (Sec. 4.2).

    Q [nq,Hq,d] and K [nkv,Hkv,d] enter as they are (no rotation); key j is visible to query q iff
    k_pos[j] <= q_pos[q].  Returns fp64 [nq,Hq,d].
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    qp, kp = _i32(q_pos), _i32(k_pos)
    sl = _f64(slopes)
    nq, Hq, d = Q.shape
    nkv, Hkv, d2 = K.shape
    assert d == d2 and V.shape == K.shape and Hq % Hkv == 0 and sl.shape == (Hq,)
    assert qp.shape == (nq,) and kp.shape == (nkv,)
    out = np.zeros((nq, Hq, d), dtype=np.float64)
    _load().orc_attn_alibi(_ptr(Q), _ptr(qp), nq, _ptr(K), _ptr(V), _ptr(kp), nkv, Hq, Hkv, d, _ptr(sl), _ptr(out))
    return out


def full_masked(Q_raw, K_raw, V, pos, module_of, base: float = 10000.0):
    """One full pass over the whole prompt under the module-local mask (Sec. 3.1/3.3).

    Returns (out [N,Hq,d], K_enc [N,Hkv,d]).
    """
    Q, K, V = _f64(Q_raw), _f64(K_raw), _f64(V)
    p, m = _i32(pos), _i32(module_of)
    N, Hq, d = Q.shape
    _, Hkv, _ = K.shape
    assert K.shape == V.shape == (N, Hkv, d) and p.shape == m.shape == (N,)
    out = np.zeros((N, Hq, d), dtype=np.float64)
    K_enc = np.zeros((N, Hkv, d), dtype=np.float64)
    _load().orc_full_masked(_ptr(Q), _ptr(K), _ptr(V), _ptr(p), _ptr(m), N, Hq, Hkv, d, float(base),
                            _ptr(out), _ptr(K_enc))
    return out, K_enc


POS_NONE = 2 ** 31 - 1   # position ID of a buffer row that holds no token (never visible)


def fill_param(K, V, pos, row0: int, length: int, K_arg_raw, V_arg, base: float = 10000.0):
    """Supply an argument to a parameter whose placeholder rows are [row0, row0+length) of an
    assembled fp64 buffer (Sec. 3.3): returns new (K, V, pos); see orc_fill_param."""
    K = np.array(_f64(K), copy=True)
    V = np.array(_f64(V), copy=True)
    pos = np.array(_i32(pos), copy=True)
    ka, va = _f64(K_arg_raw), _f64(V_arg)
    assert K.ndim == 3 and V.shape == K.shape and ka.shape == va.shape and ka.shape[1:] == K.shape[1:]
    assert 0 <= row0 and row0 + length <= K.shape[0]
    rc = _load().orc_fill_param(_ptr(K), _ptr(V), _ptr(pos), int(row0), int(length), _ptr(ka), _ptr(va),
                                int(ka.shape[0]), int(K.shape[1]), int(K.shape[2]), float(base))
    if rc != 0:
        raise ValueError("argument longer than the parameter")
    return K, V, pos


def resolve_scaffolds(import_ids: Sequence[int], scaffolds: Sequence[tuple]) -> list:
    """Scaffolding (Sec. 3.3, "attention masking effect"): a scaffold is a set of modules that was also encoded
    jointly, so that its members share one attention span.  When a prompt imports every member of a
    scaffold, the jointly encoded states override the members' own.

    scaffolds: sequence of (member_ids, override_ids), override_ids[i] naming the stored states that stand in
    for member_ids[i].  Returns the import list with each overridden id replaced where it stood.  Scaffolds
    are taken in the order given; one that would touch a member an earlier scaffold has already overridden
    is skipped (the paper does not say; first complete scaffold wins).
    """
    ids = list(import_ids)
    imported = set(ids)
    taken = set()
    for members, overrides in scaffolds:
        assert len(members) == len(overrides) and len(members) > 0
        if all(m in imported for m in members) and not any(m in taken for m in members):
            for m, o in zip(members, overrides):
                ids = [o if x == m else x for x in ids]
                taken.add(m)
    return ids


def bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """K+V bytes one cached token occupies over all layers (Table 2's closed form)."""
    return int(_load().orc_bytes_per_token(n_layers, n_kv_heads, head_dim, elem_bytes))
