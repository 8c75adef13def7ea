"""ctypes binding of ``libpromptcache.so`` (see ``include/promptcache.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Torch tensors are used as device memory (``data_ptr()``) and for the
current stream; nothing here computes.  If the shared library is missing the
import of a symbol raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpromptcache.so")

PC_F32, PC_BF16 = 0, 1

EXPORTS = [
    "pc_create", "pc_destroy", "pc_strerror", "pc_store_module", "pc_assemble_kv", "pc_prefill_attn",
    "pc_rope", "pc_append_kv", "pc_assemble_kv_batched", "pc_append_kv_batched", "pc_assemble_append_kv_batched",
    "pc_prefill_attn_batched", "pc_prefill_attn_shared_batched",
    "pc_schema_layout", "pc_uncached_positions", "pc_check_selection", "pc_bytes_per_token",
    "pc_module_info", "pc_pool_usage", "pc_last_attn_launch", "pc_profile_enable", "pc_profile_read",
    "pc_profile_read_each", "pc_set_module_params", "pc_fill_params",
    "pc_host_pool_reserve", "pc_store_module_host", "pc_set_host_copy_mode", "pc_set_attn_kernel", "pc_set_alibi", "pc_alibi_slopes",
    "pc_define_scaffold", "pc_resolve_scaffolds", "pc_calib_copy", "pc_calib_mfma",
    "pc_append_rotate_batched", "pc_assemble_append_rotate_batched", "pc_prefill_attn_rotated_batched",
    "pc_prefill_attn_shared_rotated_batched", "pc_prefill_attn_static", "pc_assemble_kv_layers", "pc_plan_stats",
]
PC_STATIC_SCRATCH_BYTES = 32 << 20
PROF_GATHER, PROF_APPEND, PROF_ATTN, PROF_COMBINE, PROF_ROPE = range(5)
PC_POS_NONE = 0x7FFFFFFF
PC_HOST_READ_KERNEL, PC_HOST_COPY_ENGINE = 0, 1
PC_ATTN_AUTO, PC_ATTN_REGISTER_STAGED = 0, 1


class PcConfig(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int), ("n_q_heads", ctypes.c_int), ("n_kv_heads", ctypes.c_int),
        ("head_dim", ctypes.c_int), ("dtype", ctypes.c_int), ("rope_base", ctypes.c_double),
        ("max_pos", ctypes.c_int), ("pool_bytes", ctypes.c_size_t), ("scratch_bytes", ctypes.c_size_t),
    ]


class PcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Open the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2311_04934_amd.build` (hipcc, gfx950)")
    L = ctypes.CDLL(LIB_PATH)
    i, vp, ip = ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)
    L.pc_create.argtypes = [ctypes.POINTER(PcConfig), ctypes.POINTER(vp)]
    L.pc_destroy.argtypes = [vp]
    L.pc_strerror.argtypes = [i]
    L.pc_strerror.restype = ctypes.c_char_p
    L.pc_store_module.argtypes = [vp, i, i, vp, vp, i, i, vp]
    L.pc_assemble_kv.argtypes = [vp, i, vp, i, vp, vp, vp, i, ip, vp]
    L.pc_prefill_attn.argtypes = [vp, i, vp, vp, i, vp, vp, vp, i, vp, vp]
    L.pc_prefill_attn_static.argtypes = [vp, i, vp, vp, i, vp, vp, vp, i, vp, vp]
    L.pc_rope.argtypes = [vp, vp, i, i, vp, vp]
    L.pc_append_kv.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp, i, i, vp]
    L.pc_assemble_kv_batched.argtypes = [vp, i, vp, vp, i, vp, vp, vp, vp, vp, vp]
    L.pc_assemble_kv_layers.argtypes = [vp, i, i, vp, vp, i, vp, vp, vp, vp, vp, vp]
    L.pc_plan_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_long), ctypes.POINTER(ctypes.c_long), ctypes.POINTER(ctypes.c_long)]
    L.pc_append_kv_batched.argtypes = [vp, i, vp, vp, vp, vp, i, vp, vp, vp, vp, vp, vp]
    L.pc_assemble_append_kv_batched.argtypes = [vp, i, vp, vp, i, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.pc_prefill_attn_batched.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp, vp, vp, vp, vp]
    L.pc_prefill_attn_shared_batched.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp, vp, vp, vp]
    L.pc_host_pool_reserve.argtypes = [vp, ctypes.c_size_t]
    L.pc_store_module_host.argtypes = [vp, i, i, vp, vp, i, i]
    L.pc_set_host_copy_mode.argtypes = [vp, i]
    L.pc_set_attn_kernel.argtypes = [vp, i]
    L.pc_set_alibi.argtypes = [vp, vp]
    L.pc_alibi_slopes.argtypes = [i, vp]
    L.pc_define_scaffold.argtypes = [vp, i, vp, vp]
    L.pc_resolve_scaffolds.argtypes = [i, vp, i, vp, vp, vp, vp]
    L.pc_calib_copy.argtypes = [vp, ctypes.c_size_t, i, ctypes.POINTER(ctypes.c_double)]
    L.pc_calib_mfma.argtypes = [vp, i, ctypes.POINTER(ctypes.c_double)]
    L.pc_append_rotate_batched.argtypes = [vp, i, vp, vp, vp, vp, vp, i, vp, vp, vp, vp, vp, vp, vp]
    L.pc_assemble_append_rotate_batched.argtypes = [vp, i, vp, vp, i, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.pc_prefill_attn_rotated_batched.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp, vp, vp, vp, vp]
    L.pc_prefill_attn_shared_rotated_batched.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp, vp, vp, vp]
    L.pc_set_module_params.argtypes = [vp, i, i, vp, vp]
    L.pc_fill_params.argtypes = [vp, i, vp, i, i, vp, vp, vp, vp, vp, vp, vp, vp, i, vp]
    L.pc_schema_layout.argtypes = [i, vp, vp, vp]
    L.pc_schema_layout.restype = ctypes.c_long
    L.pc_uncached_positions.argtypes = [i, i, i, vp]
    L.pc_check_selection.argtypes = [i, vp, vp, i]
    L.pc_bytes_per_token.argtypes = [i, i, i, i]
    L.pc_bytes_per_token.restype = ctypes.c_long
    L.pc_module_info.argtypes = [vp, i, i, ip, ip]
    L.pc_pool_usage.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    L.pc_last_attn_launch.argtypes = [vp, ip, ip, ip]
    L.pc_profile_enable.argtypes = [vp, i]
    L.pc_profile_read.argtypes = [vp, i, ip, ctypes.POINTER(ctypes.c_double)]
    L.pc_profile_read_each.argtypes = [vp, i, vp, i, ip, ctypes.POINTER(ctypes.c_double)]
    for name in EXPORTS:
        fn = getattr(L, name)
        if name not in ("pc_strerror", "pc_schema_layout", "pc_bytes_per_token"):
            fn.restype = ctypes.c_int
    _lib = L
    return L


def pc_resolve_scaffolds(import_ids: Sequence[int], scaffolds: Sequence[tuple]) -> List[int]:
    """scaffolds: sequence of (member_ids, override_ids); returns the import list with scaffolds applied."""
    ids = _ints(import_ids)
    offs = _ints(np.concatenate([[0], np.cumsum([len(m) for m, _ in scaffolds])]))
    mem = _ints([x for m, _ in scaffolds for x in m])
    ovr = _ints([x for _, o in scaffolds for x in o])
    out = np.zeros(max(len(ids), 1), dtype=np.intc)
    _check(lib().pc_resolve_scaffolds(len(ids), _np_ptr(ids), len(scaffolds), _np_ptr(offs), _np_ptr(mem), _np_ptr(ovr),
                                      _np_ptr(out)), "pc_resolve_scaffolds")
    return [int(x) for x in out[:len(ids)]]


def pc_alibi_slopes(n_heads: int) -> np.ndarray:
    out = np.zeros(max(int(n_heads), 1), dtype=np.float32)
    _check(lib().pc_alibi_slopes(int(n_heads), _np_ptr(out)), "pc_alibi_slopes")
    return out[:n_heads]


def strerror(status: int) -> str:
    return lib().pc_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise PcError(status, where)


def _ints(a: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.intc))


def _np_ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dev(t) -> Optional[int]:
    """Device pointer of a torch tensor (None passes NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ------------------------------------------------------------------ host integer helpers
def pc_schema_layout(sizes: Sequence[int], union_ids: Optional[Sequence[int]] = None) -> Tuple[List[int], int]:
    n = len(sizes)
    s = _ints(sizes)
    u = _ints(union_ids if union_ids is not None else [-1] * n)
    out = np.zeros(max(n, 1), dtype=np.intc)
    span = lib().pc_schema_layout(n, _np_ptr(s), _np_ptr(u), _np_ptr(out))
    if span < 0:
        raise PcError(int(span), "pc_schema_layout")
    return [int(x) for x in out[:n]], int(span)


def pc_uncached_positions(prev_start: int, prev_len: int, n_tokens: int) -> np.ndarray:
    pos = np.zeros(n_tokens, dtype=np.int32)
    _check(lib().pc_uncached_positions(prev_start, prev_len, n_tokens, _np_ptr(pos)), "pc_uncached_positions")
    return pos


def pc_check_selection(starts: Sequence[int], lens: Sequence[int], max_pos: int) -> int:
    s, l = _ints(starts), _ints(lens)
    return int(lib().pc_check_selection(len(s), _np_ptr(s), _np_ptr(l), int(max_pos)))


def pc_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, dtype: int) -> int:
    return int(lib().pc_bytes_per_token(n_layers, n_kv_heads, head_dim, dtype))


# ------------------------------------------------------------------ context
class PromptCache:
    """Owner of a ``pc_ctx``.  Methods mirror the C entry points one to one."""

    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int,
                 rope_base: float = 10000.0, max_pos: int = 16384, pool_bytes: int = 1 << 30,
                 scratch_bytes: int = 0):
        self.cfg = PcConfig(n_layers, n_q_heads, n_kv_heads, head_dim, dtype, rope_base, max_pos,
                            pool_bytes, scratch_bytes)
        self._ctx = ctypes.c_void_p()
        _check(lib().pc_create(ctypes.byref(self.cfg), ctypes.byref(self._ctx)), "pc_create")

    @classmethod
    def for_workload(cls, w, pool_bytes: Optional[int] = None, n_layers: Optional[int] = None, **kw):
        L = n_layers if n_layers is not None else w.n_layers
        if pool_bytes is None:
            rows = sum(w.sizes[m] for m in w.used_module_ids())
            pool_bytes = L * (2 * rows * w.row_bytes + 512 * len(w.sizes)) + (1 << 20)
        return cls(L, w.n_q_heads, w.n_kv_heads, w.head_dim, PC_F32 if w.dtype == "f32" else PC_BF16,
                   w.rope_base, w.max_pos, pool_bytes, **kw)

    def close(self) -> None:
        if self._ctx:
            lib().pc_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the three calls of the path
    def pc_store_module(self, layer: int, module_id: int, K, V, start_pos: int, stream=None) -> None:
        n = int(K.shape[0])
        _check(lib().pc_store_module(self._ctx, layer, module_id, _dev(K), _dev(V), n, start_pos, _stream(stream)),
               "pc_store_module")

    def pc_assemble_kv(self, layer: int, module_ids: Sequence[int], out_K, out_V, out_pos,
                       capacity_tokens: Optional[int] = None, stream=None) -> int:
        ids = _ints(module_ids)
        cap = int(out_K.shape[0]) if capacity_tokens is None else capacity_tokens
        n_out = ctypes.c_int(0)
        _check(lib().pc_assemble_kv(self._ctx, layer, _np_ptr(ids), len(ids), _dev(out_K), _dev(out_V), _dev(out_pos),
                                    cap, ctypes.byref(n_out), _stream(stream)), "pc_assemble_kv")
        return n_out.value

    def pc_prefill_attn(self, layer: int, Q_new, q_pos, asm_K, asm_V, asm_pos, n_kv: int, out, stream=None) -> None:
        n_q = int(Q_new.shape[0])
        _check(lib().pc_prefill_attn(self._ctx, layer, _dev(Q_new), _dev(q_pos), n_q, _dev(asm_K), _dev(asm_V),
                                     _dev(asm_pos), n_kv, _dev(out), _stream(stream)), "pc_prefill_attn")

    def pc_prefill_attn_static(self, layer: int, Q_new, q_pos, asm_K, asm_V, asm_pos, n_kv: int, out, stream=None) -> None:
        n_q = int(Q_new.shape[0])
        _check(lib().pc_prefill_attn_static(self._ctx, layer, _dev(Q_new), _dev(q_pos), n_q, _dev(asm_K), _dev(asm_V),
                                            _dev(asm_pos), n_kv, _dev(out), _stream(stream)), "pc_prefill_attn_static")

    # -- supporting calls
    def pc_rope(self, x, pos, stream=None) -> None:
        _check(lib().pc_rope(self._ctx, _dev(x), int(x.shape[0]), int(x.shape[1]), _dev(pos), _stream(stream)), "pc_rope")

    def pc_append_kv(self, layer: int, K_new_raw, V_new, q_pos, asm_K, asm_V, asm_pos, n_kv_before: int,
                     capacity_tokens: Optional[int] = None, stream=None) -> None:
        cap = int(asm_K.shape[0]) if capacity_tokens is None else capacity_tokens
        _check(lib().pc_append_kv(self._ctx, layer, _dev(K_new_raw), _dev(V_new), _dev(q_pos), int(K_new_raw.shape[0]),
                                  _dev(asm_K), _dev(asm_V), _dev(asm_pos), n_kv_before, cap, _stream(stream)),
               "pc_append_kv")

    # -- batched
    def pc_assemble_kv_batched(self, layer: int, module_ids: Sequence[Sequence[int]], out_K, out_V, out_pos,
                               kv_offsets: Sequence[int], stream=None) -> List[int]:
        flat = _ints([m for ids in module_ids for m in ids])
        offs = _ints(np.concatenate([[0], np.cumsum([len(ids) for ids in module_ids])]))
        kvo = _ints(kv_offsets)
        B = len(module_ids)
        assert len(kvo) == B + 1
        n_out = np.zeros(max(B, 1), dtype=np.intc)
        _check(lib().pc_assemble_kv_batched(self._ctx, layer, _np_ptr(flat), _np_ptr(offs), B, _dev(out_K), _dev(out_V),
                                            _dev(out_pos), _np_ptr(kvo), _np_ptr(n_out), _stream(stream)),
               "pc_assemble_kv_batched")
        return [int(x) for x in n_out[:B]]

    def pc_assemble_kv_layers(self, first_layer: int, module_ids: Sequence[Sequence[int]], out_K: Sequence, out_V: Sequence,
                              out_pos: Sequence, kv_offsets: Sequence[int], stream=None) -> List[int]:
        """out_K/out_V/out_pos: one device tensor per layer, layers first_layer .. first_layer+len(out_K)-1."""
        flat = _ints([m for ids in module_ids for m in ids])
        offs = _ints(np.concatenate([[0], np.cumsum([len(ids) for ids in module_ids])]))
        kvo = _ints(kv_offsets)
        B, L = len(module_ids), len(out_K)
        assert len(kvo) == B + 1 and len(out_V) == L and len(out_pos) == L
        ptrs = [(ctypes.c_void_p * max(L, 1))(*[_dev(t) for t in ts]) for ts in (out_K, out_V, out_pos)]
        n_out = np.zeros(max(B, 1), dtype=np.intc)
        _check(lib().pc_assemble_kv_layers(self._ctx, first_layer, L, _np_ptr(flat), _np_ptr(offs), B, ptrs[0], ptrs[1],
                                           ptrs[2], _np_ptr(kvo), _np_ptr(n_out), _stream(stream)),
               "pc_assemble_kv_layers")
        return [int(x) for x in n_out[:B]]

    def pc_append_kv_batched(self, layer: int, K_new_raw, V_new, q_pos, q_offsets: Sequence[int], asm_K, asm_V,
                             asm_pos, kv_offsets: Sequence[int], kv_lens: Sequence[int], stream=None) -> None:
        qo, kvo, kvl = _ints(q_offsets), _ints(kv_offsets), _ints(kv_lens)
        B = len(kvl)
        assert len(qo) == B + 1 and len(kvo) == B + 1
        _check(lib().pc_append_kv_batched(self._ctx, layer, _dev(K_new_raw), _dev(V_new), _dev(q_pos), _np_ptr(qo), B,
                                          _dev(asm_K), _dev(asm_V), _dev(asm_pos), _np_ptr(kvo), _np_ptr(kvl),
                                          _stream(stream)), "pc_append_kv_batched")

    def pc_assemble_append_kv_batched(self, layer: int, module_ids: Sequence[Sequence[int]], K_new_raw, V_new, q_pos,
                                      q_offsets: Sequence[int], out_K, out_V, out_pos, kv_offsets: Sequence[int],
                                      stream=None) -> List[int]:
        flat = _ints([m for ids in module_ids for m in ids])
        offs = _ints(np.concatenate([[0], np.cumsum([len(ids) for ids in module_ids])]))
        qo, kvo = _ints(q_offsets), _ints(kv_offsets)
        B = len(module_ids)
        assert len(kvo) == B + 1 and len(qo) == B + 1
        n_out = np.zeros(max(B, 1), dtype=np.intc)
        _check(lib().pc_assemble_append_kv_batched(self._ctx, layer, _np_ptr(flat), _np_ptr(offs), B, _dev(K_new_raw),
                                                   _dev(V_new), _dev(q_pos), _np_ptr(qo), _dev(out_K), _dev(out_V),
                                                   _dev(out_pos), _np_ptr(kvo), _np_ptr(n_out), _stream(stream)),
               "pc_assemble_append_kv_batched")
        return [int(x) for x in n_out[:B]]

    def pc_prefill_attn_batched(self, layer: int, Q_new, q_pos, q_offsets: Sequence[int], asm_K, asm_V, asm_pos,
                                kv_offsets: Sequence[int], kv_lens: Sequence[int], out, stream=None) -> None:
        qo, kvo, kvl = _ints(q_offsets), _ints(kv_offsets), _ints(kv_lens)
        B = len(kvl)
        assert len(qo) == B + 1 and len(kvo) == B + 1
        _check(lib().pc_prefill_attn_batched(self._ctx, layer, _dev(Q_new), _dev(q_pos), _np_ptr(qo), B, _dev(asm_K),
                                             _dev(asm_V), _dev(asm_pos), _np_ptr(kvo), _np_ptr(kvl), _dev(out),
                                             _stream(stream)), "pc_prefill_attn_batched")

    def pc_prefill_attn_shared_batched(self, layer: int, Q_new, q_pos, q_offsets: Sequence[int],
                                       module_ids: Sequence[Sequence[int]], K_tail, V_tail, out, stream=None) -> None:
        qo = _ints(q_offsets)
        flat = _ints([m for ids in module_ids for m in ids])
        offs = _ints(np.concatenate([[0], np.cumsum([len(ids) for ids in module_ids])]))
        B = len(module_ids)
        assert len(qo) == B + 1
        _check(lib().pc_prefill_attn_shared_batched(self._ctx, layer, _dev(Q_new), _dev(q_pos), _np_ptr(qo), B,
                                                    _np_ptr(flat), _np_ptr(offs), _dev(K_tail), _dev(V_tail), _dev(out),
                                                    _stream(stream)), "pc_prefill_attn_shared_batched")

    def pc_host_pool_reserve(self, n_bytes: int) -> None:
        _check(lib().pc_host_pool_reserve(self._ctx, int(n_bytes)), "pc_host_pool_reserve")

    def pc_store_module_host(self, layer: int, module_id: int, K_host, V_host, start_pos: int) -> None:
        """K_host / V_host: contiguous CPU torch tensors [n_tokens, n_kv_heads, head_dim]."""
        assert not K_host.is_cuda and not V_host.is_cuda and K_host.is_contiguous() and V_host.is_contiguous()
        assert K_host.shape == V_host.shape
        n = int(K_host.shape[0])
        _check(lib().pc_store_module_host(self._ctx, layer, int(module_id), K_host.data_ptr() if n else None,
                                          V_host.data_ptr() if n else None, n, int(start_pos)), "pc_store_module_host")

    def pc_set_host_copy_mode(self, mode: int) -> None:
        _check(lib().pc_set_host_copy_mode(self._ctx, int(mode)), "pc_set_host_copy_mode")

    def pc_set_attn_kernel(self, which: int) -> None:
        _check(lib().pc_set_attn_kernel(self._ctx, int(which)), "pc_set_attn_kernel")

    # -- Q rotated once per token (in the append launch) instead of in every attention workgroup
    def pc_append_rotate_batched(self, layer: int, K_new_raw, V_new, Q_new, q_pos, q_offsets: Sequence[int], asm_K, asm_V,
                                 asm_pos, kv_offsets: Sequence[int], kv_lens: Sequence[int], Q_rot, stream=None) -> None:
        qo, kvo, kvl = _ints(q_offsets), _ints(kv_offsets), _ints(kv_lens)
        B = len(kvl)
        assert len(qo) == B + 1 and len(kvo) == B + 1
        _check(lib().pc_append_rotate_batched(self._ctx, layer, _dev(K_new_raw), _dev(V_new), _dev(Q_new), _dev(q_pos),
                                              _np_ptr(qo), B, _dev(asm_K), _dev(asm_V), _dev(asm_pos), _np_ptr(kvo),
                                              _np_ptr(kvl), _dev(Q_rot), _stream(stream)), "pc_append_rotate_batched")

    def pc_assemble_append_rotate_batched(self, layer: int, module_ids: Sequence[Sequence[int]], K_new_raw, V_new, Q_new,
                                          q_pos, q_offsets: Sequence[int], out_K, out_V, out_pos,
                                          kv_offsets: Sequence[int], Q_rot, stream=None) -> List[int]:
        flat = _ints([m for ids in module_ids for m in ids])
        offs = _ints(np.concatenate([[0], np.cumsum([len(ids) for ids in module_ids])]))
        qo, kvo = _ints(q_offsets), _ints(kv_offsets)
        B = len(module_ids)
        assert len(qo) == B + 1 and len(kvo) == B + 1
        n_out = np.zeros(max(B, 1), dtype=np.intc)
        _check(lib().pc_assemble_append_rotate_batched(self._ctx, layer, _np_ptr(flat), _np_ptr(offs), B, _dev(K_new_raw),
                                                       _dev(V_new), _dev(Q_new), _dev(q_pos), _np_ptr(qo), _dev(out_K),
                                                       _dev(out_V), _dev(out_pos), _np_ptr(kvo), _np_ptr(n_out), _dev(Q_rot),
                                                       _stream(stream)), "pc_assemble_append_rotate_batched")
        return [int(x) for x in n_out[:B]]

    def pc_prefill_attn_rotated_batched(self, layer: int, Q_rot, q_pos, q_offsets: Sequence[int], asm_K, asm_V, asm_pos,
                                        kv_offsets: Sequence[int], kv_lens: Sequence[int], out, stream=None) -> None:
        qo, kvo, kvl = _ints(q_offsets), _ints(kv_offsets), _ints(kv_lens)
        B = len(kvl)
        assert len(qo) == B + 1 and len(kvo) == B + 1
        _check(lib().pc_prefill_attn_rotated_batched(self._ctx, layer, _dev(Q_rot), _dev(q_pos), _np_ptr(qo), B, _dev(asm_K),
                                                     _dev(asm_V), _dev(asm_pos), _np_ptr(kvo), _np_ptr(kvl), _dev(out),
                                                     _stream(stream)), "pc_prefill_attn_rotated_batched")

    def pc_prefill_attn_shared_rotated_batched(self, layer: int, Q_rot, q_pos, q_offsets: Sequence[int],
                                               module_ids: Sequence[Sequence[int]], K_tail, V_tail, out, stream=None) -> None:
        qo = _ints(q_offsets)
        flat = _ints([m for ids in module_ids for m in ids])
        offs = _ints(np.concatenate([[0], np.cumsum([len(ids) for ids in module_ids])]))
        B = len(module_ids)
        assert len(qo) == B + 1
        _check(lib().pc_prefill_attn_shared_rotated_batched(self._ctx, layer, _dev(Q_rot), _dev(q_pos), _np_ptr(qo), B,
                                                            _np_ptr(flat), _np_ptr(offs), _dev(K_tail), _dev(V_tail),
                                                            _dev(out), _stream(stream)), "pc_prefill_attn_shared_rotated_batched")

    def pc_calib_copy(self, n_bytes: int, repeats: int = 10) -> float:
        v = ctypes.c_double(0.0)
        _check(lib().pc_calib_copy(self._ctx, int(n_bytes), int(repeats), ctypes.byref(v)), "pc_calib_copy")
        return v.value

    def pc_calib_mfma(self, iters: int = 4000) -> float:
        v = ctypes.c_double(0.0)
        _check(lib().pc_calib_mfma(self._ctx, int(iters), ctypes.byref(v)), "pc_calib_mfma")
        return v.value

    def pc_define_scaffold(self, member_ids: Sequence[int], override_ids: Sequence[int]) -> None:
        m, o = _ints(member_ids), _ints(override_ids)
        assert len(m) == len(o)
        _check(lib().pc_define_scaffold(self._ctx, len(m), _np_ptr(m), _np_ptr(o)), "pc_define_scaffold")

    def pc_set_alibi(self, slopes) -> None:
        """slopes: n_q_heads floats (host), or None to return to rotary encoding."""
        if slopes is None:
            _check(lib().pc_set_alibi(self._ctx, None), "pc_set_alibi")
            return
        a = np.ascontiguousarray(np.asarray(slopes, dtype=np.float32))
        _check(lib().pc_set_alibi(self._ctx, _np_ptr(a)), "pc_set_alibi")

    def pc_set_module_params(self, module_id: int, offsets: Sequence[int], lens: Sequence[int]) -> None:
        o, l = _ints(offsets), _ints(lens)
        assert len(o) == len(l)
        _check(lib().pc_set_module_params(self._ctx, int(module_id), len(o), _np_ptr(o), _np_ptr(l)),
               "pc_set_module_params")

    def pc_fill_params(self, layer: int, module_ids: Sequence[int], arg_module: Sequence[int],
                       arg_param: Sequence[int], arg_offsets: Sequence[int], K_arg_raw, V_arg, asm_K, asm_V, asm_pos,
                       stream=None) -> None:
        ids, am, ap, ao = _ints(module_ids), _ints(arg_module), _ints(arg_param), _ints(arg_offsets)
        assert len(am) == len(ap) and len(ao) == len(am) + 1
        _check(lib().pc_fill_params(self._ctx, layer, _np_ptr(ids), len(ids), len(am), _np_ptr(am), _np_ptr(ap),
                                    _np_ptr(ao), _dev(K_arg_raw), _dev(V_arg), _dev(asm_K), _dev(asm_V), _dev(asm_pos),
                                    int(asm_pos.shape[0]), _stream(stream)), "pc_fill_params")

    # -- queries
    def pc_module_info(self, layer: int, module_id: int) -> Tuple[int, int]:
        n, s = ctypes.c_int(0), ctypes.c_int(0)
        _check(lib().pc_module_info(self._ctx, layer, module_id, ctypes.byref(n), ctypes.byref(s)), "pc_module_info")
        return n.value, s.value

    def pc_plan_stats(self) -> Tuple[int, int, int]:
        """(calls served from a kept plan, calls that planned, host heap allocations of the planning code so far)."""
        h, m, a = ctypes.c_long(0), ctypes.c_long(0), ctypes.c_long(0)
        _check(lib().pc_plan_stats(self._ctx, ctypes.byref(h), ctypes.byref(m), ctypes.byref(a)), "pc_plan_stats")
        return h.value, m.value, a.value

    def pc_pool_usage(self) -> Tuple[int, int]:
        u, t = ctypes.c_size_t(0), ctypes.c_size_t(0)
        _check(lib().pc_pool_usage(self._ctx, ctypes.byref(u), ctypes.byref(t)), "pc_pool_usage")
        return u.value, t.value

    def pc_last_attn_launch(self) -> Tuple[int, int, int]:
        a, b, c = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
        _check(lib().pc_last_attn_launch(self._ctx, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
               "pc_last_attn_launch")
        return a.value, b.value, c.value

    def pc_profile_enable(self, max_records_per_kind: int) -> None:
        _check(lib().pc_profile_enable(self._ctx, int(max_records_per_kind)), "pc_profile_enable")

    def pc_profile_read(self, kind: int) -> Tuple[int, float]:
        n, ms = ctypes.c_int(0), ctypes.c_double(0.0)
        _check(lib().pc_profile_read(self._ctx, int(kind), ctypes.byref(n), ctypes.byref(ms)), "pc_profile_read")
        return n.value, ms.value

    def pc_profile_read_each(self, kind: int, capacity: int) -> np.ndarray:
        """Durations (ms) of the recorded launches of one kind, in launch order."""
        buf = np.zeros(max(capacity, 1), dtype=np.float32)
        n, ms = ctypes.c_int(0), ctypes.c_double(0.0)
        _check(lib().pc_profile_read_each(self._ctx, int(kind), _np_ptr(buf), int(capacity), ctypes.byref(n),
                                          ctypes.byref(ms)), "pc_profile_read_each")
        return buf[:min(n.value, capacity)].copy()
