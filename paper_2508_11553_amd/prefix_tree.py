"""ctypes wrapper of the host-side session prefix tree (sd_tree_* in the C ABI)."""
from __future__ import annotations

import ctypes

import numpy as np

from . import binding as sd


def _lib():
    L = sd.load()
    if not getattr(L, "_tree_ready", False):
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.sd_tree_create.restype, L.sd_tree_create.argtypes = vp, [i32]
        L.sd_tree_destroy.restype, L.sd_tree_destroy.argtypes = None, [vp]
        L.sd_tree_pages_in_use.restype, L.sd_tree_pages_in_use.argtypes = i32, [vp]
        L.sd_tree_match.restype, L.sd_tree_match.argtypes = i32, [vp, vp, vp, i32]
        L.sd_tree_insert.restype, L.sd_tree_insert.argtypes = i32, [vp, vp, vp, i32, vp]
        L.sd_tree_release.restype, L.sd_tree_release.argtypes = ctypes.c_int, [vp, i32]
        L.sd_tree_fork.restype, L.sd_tree_fork.argtypes = i32, [vp, i32, vp, vp]
        L.sd_tree_append.restype, L.sd_tree_append.argtypes = ctypes.c_int, [vp, i32, i32, ctypes.c_uint32, vp, vp]
        L.sd_tree_length.restype, L.sd_tree_length.argtypes = i32, [vp, i32]
        L.sd_tree_block_table.restype, L.sd_tree_block_table.argtypes = i32, [vp, i32, vp, i32]
        L.sd_tree_token_at.restype, L.sd_tree_token_at.argtypes = ctypes.c_int, [vp, i32, i32, vp, vp]
        L.sd_tree_batch_groups.restype, L.sd_tree_batch_groups.argtypes = i32, [vp, vp, i32, vp, vp]
        L._tree_ready = True
    return L


def _arr(a, dtype):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


class PrefixTree:
    def __init__(self, num_pages: int):
        self._h = _lib().sd_tree_create(int(num_pages))
        if not self._h:
            raise ValueError("sd_tree_create failed")

    def close(self):
        if self._h:
            _lib().sd_tree_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def pages_in_use(self) -> int:
        return int(_lib().sd_tree_pages_in_use(self._h))

    def match(self, tokens, versions=None) -> int:
        t, tp = _arr(tokens, np.int32)
        v, vp = _arr(versions, np.uint32)
        return int(_lib().sd_tree_match(self._h, tp, vp, len(t)))

    def insert(self, tokens, versions=None):
        """-> (trajectory id, tokens whose pages already existed)."""
        t, tp = _arr(tokens, np.int32)
        v, vp = _arr(versions, np.uint32)
        m = ctypes.c_int32(0)
        rc = int(_lib().sd_tree_insert(self._h, tp, vp, len(t), ctypes.byref(m)))
        if rc < 0:
            raise sd.SeamDecodeError(rc, "sd_tree_insert")
        return rc, int(m.value)

    def release(self, traj: int):
        rc = int(_lib().sd_tree_release(self._h, int(traj)))
        if rc:
            raise sd.SeamDecodeError(rc, "sd_tree_release")

    def fork(self, traj: int):
        """-> (new trajectory id, page to copy from, page to copy to); the pages are -1 if nothing is to be copied."""
        src, dst = ctypes.c_int32(-1), ctypes.c_int32(-1)
        rc = int(_lib().sd_tree_fork(self._h, int(traj), ctypes.byref(src), ctypes.byref(dst)))
        if rc < 0:
            raise sd.SeamDecodeError(rc, "sd_tree_fork")
        return rc, int(src.value), int(dst.value)

    def append(self, traj: int, token: int, version: int = 0):
        """One more token; -> (page, slot) its K/V rows go to."""
        page, slot = ctypes.c_int32(-1), ctypes.c_int32(-1)
        rc = int(_lib().sd_tree_append(self._h, int(traj), int(token), int(version), ctypes.byref(page),
                                       ctypes.byref(slot)))
        if rc:
            raise sd.SeamDecodeError(rc, "sd_tree_append")
        return int(page.value), int(slot.value)

    def length(self, traj: int) -> int:
        return int(_lib().sd_tree_length(self._h, int(traj)))

    def block_table(self, traj: int) -> np.ndarray:
        n = int(_lib().sd_tree_block_table(self._h, int(traj), None, 0))
        if n < 0:
            raise sd.SeamDecodeError(n, "sd_tree_block_table")
        out = np.zeros(max(n, 1), np.int32)
        _lib().sd_tree_block_table(self._h, int(traj), out.ctypes.data_as(ctypes.c_void_p), n)
        return out[:n]

    def token_at(self, traj: int, pos: int):
        tok, ver = ctypes.c_int32(0), ctypes.c_uint32(0)
        rc = int(_lib().sd_tree_token_at(self._h, int(traj), int(pos), ctypes.byref(tok), ctypes.byref(ver)))
        if rc:
            raise sd.SeamDecodeError(rc, "sd_tree_token_at")
        return int(tok.value), int(ver.value)

    def batch_groups(self, trajs):
        """-> (group_start int32[groups+1], shared_len int32[B])."""
        t, tp = _arr(trajs, np.int32)
        gs = np.zeros(len(t) + 1, np.int32)
        sh = np.zeros(max(len(t), 1), np.int32)
        ng = int(_lib().sd_tree_batch_groups(self._h, tp, len(t), gs.ctypes.data_as(ctypes.c_void_p),
                                             sh.ctypes.data_as(ctypes.c_void_p)))
        if ng < 0:
            raise sd.SeamDecodeError(ng, "sd_tree_batch_groups")
        return gs[:ng + 1], sh[:len(t)]
