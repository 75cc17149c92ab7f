"""Thin ctypes binding of include/das_drafter.h (suffix-tree drafter over a window of recent rollouts, Sec. 4.1.2).
Argument marshalling only; the index lives in csrc/das_drafter.cpp."""
import ctypes as C

import numpy as np

from .binding import lib


class DrafterError(RuntimeError):
    pass


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Drafter:
    def __init__(self, max_epochs=4):
        L = lib()
        L.das_drafter_create.argtypes = [C.c_int32, C.POINTER(C.c_void_p)]
        L.das_drafter_free.argtypes = [C.c_void_p]
        L.das_drafter_new_epoch.argtypes = [C.c_void_p]
        L.das_drafter_add.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        L.das_drafter_propose.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                          C.POINTER(C.c_int32), C.c_void_p, C.POINTER(C.c_int32)]
        L.das_drafter_size.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        self.h = C.c_void_p()
        self._chk(L.das_drafter_create(int(max_epochs), C.byref(self.h)), "das_drafter_create")

    @staticmethod
    def _chk(code, what):
        if code != 0:
            raise DrafterError(f"{what}: error {code}")

    def free(self):
        if getattr(self, "h", None):
            lib().das_drafter_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def new_epoch(self):
        self._chk(lib().das_drafter_new_epoch(self.h), "das_drafter_new_epoch")

    def add(self, tokens):
        t = _i32(tokens)
        self._chk(lib().das_drafter_add(self.h, t.ctypes.data, t.size), "das_drafter_add")

    def propose(self, ctx, k, max_match=32, min_match=1):
        """(match length, draft tokens) for the end of ctx."""
        c = _i32(ctx)
        out = np.empty(max(int(k), 1), np.int32)
        ml, nd = C.c_int32(), C.c_int32()
        self._chk(lib().das_drafter_propose(self.h, c.ctypes.data, c.size, int(max_match), int(min_match), int(k),
                                            C.byref(ml), out.ctypes.data, C.byref(nd)), "das_drafter_propose")
        return ml.value, out[:nd.value].copy()

    def size(self):
        t, n, e = C.c_int64(), C.c_int64(), C.c_int32()
        self._chk(lib().das_drafter_size(self.h, C.byref(t), C.byref(n), C.byref(e)), "das_drafter_size")
        return {"tokens": t.value, "nodes": n.value, "epochs": e.value}
