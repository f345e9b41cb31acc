"""ctypes binding of the paged activation store in libdaf.so (include/daf_store.h): same
names as the C ABI, argument marshalling only.  Host-side bookkeeping; no GPU call is made."""
import ctypes as c
from typing import List, Optional, Sequence, Tuple

from .binding import DafError, load_library

INDEX_RBTREE, INDEX_SORT = 0, 1
PLANNED, ALLOCATED, EVICTED, RELEASED = 0, 1, 2, 3

_ready = False


class _Move(c.Structure):
    _fields_ = [("id", c.c_int64), ("from_offset_bytes", c.c_int64), ("to_offset_bytes", c.c_int64),
                ("size_bytes", c.c_int64)]


def _lib():
    global _ready
    L = load_library()
    if not _ready:
        vp, i64, i32 = c.c_void_p, c.c_int64, c.c_int32
        L.daf_store_create.argtypes = [i64, i64, i64, i64, c.c_int, c.POINTER(vp)]
        L.daf_store_destroy.argtypes = [vp]
        L.daf_store_destroy.restype = None
        L.daf_store_reset.argtypes = [vp]
        L.daf_store_add.argtypes = [vp, i64, c.POINTER(i32), c.POINTER(i64), c.POINTER(i64), i32, c.c_double]
        L.daf_store_receive.argtypes = [vp, i64, c.c_double, c.POINTER(i32), c.POINTER(i64), c.POINTER(i64)]
        L.daf_store_add_many.argtypes = [vp, i64, vp, vp, vp, vp, i32, vp]
        L.daf_store_receive_many.argtypes = [vp, i64, vp, vp, vp, vp, vp]
        L.daf_store_release.argtypes = [vp, i64]
        L.daf_store_set_mem_budget.argtypes = [vp, i64, c.POINTER(_Move), i32, c.POINTER(i32)]
        L.daf_store_set_time_budget.argtypes = [vp, i64]
        L.daf_store_query.argtypes = [vp, i64, c.POINTER(i32), c.POINTER(i32), c.POINTER(i64), c.POINTER(i64)]
        L.daf_store_pop_evicted.argtypes = [vp, c.POINTER(i64), i32]
        L.daf_store_pop_evicted.restype = i32
        for name in ("daf_store_capacity_bytes", "daf_store_used_bytes", "daf_store_used_time_ns",
                     "daf_store_num_selections"):
            getattr(L, name).argtypes = [vp]
            getattr(L, name).restype = i64
        L.daf_store_validate.argtypes = [vp]
        _ready = True
    return L


def _check(status: int, where: str):
    if status != 0:
        raise DafError(status, where)


class Store:
    """Owns one daf_store_t."""

    def __init__(self, page_bytes: int, mem_budget_bytes: int, time_budget_ns: Optional[int], step_bytes: int,
                 index_kind: int = INDEX_RBTREE):
        self._h = c.c_void_p()
        self._n = 0
        _check(_lib().daf_store_create(page_bytes, mem_budget_bytes, time_budget_ns or 0, step_bytes, index_kind,
                                       c.byref(self._h)), "daf_store_create")

    def destroy(self):
        if self._h:
            _lib().daf_store_destroy(self._h)
            self._h = c.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reset(self):
        _check(_lib().daf_store_reset(self._h), "daf_store_reset")
        self._n = 0

    def add(self, act_id: int, widths: Sequence[int], bytes_per_width: Sequence[int],
            time_ns_per_width: Sequence[int], moving_avg_importance: float):
        n = len(widths)
        if not (n == len(bytes_per_width) == len(time_ns_per_width)):
            raise ValueError("widths, bytes_per_width and time_ns_per_width must have the same length")
        _check(_lib().daf_store_add(self._h, act_id, (c.c_int32 * n)(*widths), (c.c_int64 * n)(*bytes_per_width),
                                    (c.c_int64 * n)(*time_ns_per_width), n, float(moving_avg_importance)),
               "daf_store_add")
        self._n += 1

    def receive(self, act_id: int, importance: float) -> Tuple[int, int, int]:
        bits, off, size = c.c_int32(), c.c_int64(), c.c_int64()
        _check(_lib().daf_store_receive(self._h, act_id, float(importance), c.byref(bits), c.byref(off),
                                        c.byref(size)), "daf_store_receive")
        return bits.value, off.value, size.value

    def add_many(self, ids, widths: Sequence[int], bytes_per_width, time_ns_per_width, moving_avg_importance):
        """ids int64[n]; bytes_per_width, time_ns_per_width int64[n, len(widths)]; importance float64[n]."""
        import numpy as np
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        w = np.ascontiguousarray(widths, dtype=np.int32)
        by = np.ascontiguousarray(bytes_per_width, dtype=np.int64)
        tm = np.ascontiguousarray(time_ns_per_width, dtype=np.int64)
        imp = np.ascontiguousarray(moving_avg_importance, dtype=np.float64)
        if by.shape != (ids.size, w.size) or tm.shape != by.shape or imp.shape != (ids.size,):
            raise ValueError("add_many: array shapes do not match")
        _check(_lib().daf_store_add_many(self._h, ids.size, ids.ctypes.data, w.ctypes.data, by.ctypes.data,
                                         tm.ctypes.data, w.size, imp.ctypes.data), "daf_store_add_many")
        self._n += ids.size

    def receive_many(self, ids, importance):
        """Returns (bits int32[n], offset_bytes int64[n], size_bytes int64[n])."""
        import numpy as np
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        imp = np.ascontiguousarray(importance, dtype=np.float64)
        if imp.shape != ids.shape:
            raise ValueError("receive_many: array shapes do not match")
        bits = np.empty(ids.size, np.int32)
        off = np.empty(ids.size, np.int64)
        size = np.empty(ids.size, np.int64)
        _check(_lib().daf_store_receive_many(self._h, ids.size, ids.ctypes.data, imp.ctypes.data, bits.ctypes.data,
                                             off.ctypes.data, size.ctypes.data), "daf_store_receive_many")
        return bits, off, size

    def release(self, act_id: int):
        _check(_lib().daf_store_release(self._h, act_id), "daf_store_release")

    def set_mem_budget(self, mem_budget_bytes: int) -> List[Tuple[int, int, int, int]]:
        cap = max(self._n, 1)
        moves, n = (_Move * cap)(), c.c_int32()
        _check(_lib().daf_store_set_mem_budget(self._h, mem_budget_bytes, moves, cap, c.byref(n)),
               "daf_store_set_mem_budget")
        return [(m.id, m.from_offset_bytes, m.to_offset_bytes, m.size_bytes) for m in moves[:n.value]]

    def set_time_budget(self, time_budget_ns: Optional[int]):
        _check(_lib().daf_store_set_time_budget(self._h, time_budget_ns or 0), "daf_store_set_time_budget")

    def query(self, act_id: int) -> Tuple[int, int, int, int]:
        st, bits, off, size = c.c_int32(), c.c_int32(), c.c_int64(), c.c_int64()
        _check(_lib().daf_store_query(self._h, act_id, c.byref(st), c.byref(bits), c.byref(off), c.byref(size)),
               "daf_store_query")
        return st.value, bits.value, off.value, size.value

    def pop_evicted(self) -> List[int]:
        out, buf = [], (c.c_int64 * 64)()
        while True:
            n = _lib().daf_store_pop_evicted(self._h, buf, 64)
            out += list(buf[:n])
            if n < 64:
                return out

    def capacity_bytes(self) -> int:
        return _lib().daf_store_capacity_bytes(self._h)

    def used_bytes(self) -> int:
        return _lib().daf_store_used_bytes(self._h)

    def used_time_ns(self) -> int:
        return _lib().daf_store_used_time_ns(self._h)

    def num_selections(self) -> int:
        return _lib().daf_store_num_selections(self._h)

    def validate(self) -> bool:
        return _lib().daf_store_validate(self._h) == 0
