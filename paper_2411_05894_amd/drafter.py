"""ctypes binding of the host-side drafter in libsssd_verify.so (include/sssd_draft.h): same names
as the C ABI, argument marshalling only.  Host memory throughout; needs no GPU."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .binding import SssdError, lib as _base_lib

SSSD_OK = 0


class DraftParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("prefix_len", "branch_len", "max_tree_nodes", "max_samples", "max_sub_indices")] + \
               [(n, C.c_double) for n in ("input_discount", "datastore_match", "child_disc_base", "child_disc_per_match")]


_ready = False


def lib() -> C.CDLL:
    global _ready
    l = _base_lib()
    if not _ready:
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        l.sssd_draft_default_params.argtypes = [C.POINTER(DraftParams)]
        l.sssd_draft_default_params.restype = None
        l.sssd_draft_create.argtypes = [C.POINTER(DraftParams), i32, C.POINTER(vp)]
        l.sssd_draft_destroy.argtypes = [vp]
        l.sssd_draft_input_reset.argtypes = [vp, i32]
        l.sssd_draft_input_append.argtypes = [vp, i32, vp, i32]
        l.sssd_draft_datastore_add.argtypes = [vp, vp, i64]
        l.sssd_draft_propose.argtypes = [vp, i32, i32, vp, vp, C.POINTER(i32)]
        l.sssd_draft_speculation_length.argtypes = [C.c_double, C.c_double, i32, i32]
        l.sssd_draft_speculation_length.restype = i32
        l.sssd_draft_input_count.argtypes = [vp, i32, vp, i32]
        l.sssd_draft_input_count.restype = i64
        l.sssd_draft_match_input.argtypes = [vp, i32, vp]
        l.sssd_draft_match_input.restype = i32
        l.sssd_draft_datastore_lookup.argtypes = [vp, i32, vp, i32, vp, i64, C.POINTER(i64)]
        l.sssd_draft_datastore_tree.argtypes = [vp, i32, vp, vp, vp, C.POINTER(i32)]
        _ready = True
    return l


def _check(code: int, what: str) -> None:
    if code != SSSD_OK:
        raise SssdError(code, what)


def _i32(a: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def default_params() -> DraftParams:
    p = DraftParams()
    lib().sssd_draft_default_params(C.byref(p))
    return p


def sssd_draft_speculation_length(peak_flops: float, peak_bytes_per_s: float, b: int, cap: int) -> int:
    return int(lib().sssd_draft_speculation_length(peak_flops, peak_bytes_per_s, b, cap))


class Drafter:
    """Owns one sssd_drafter handle."""

    def __init__(self, params: Optional[DraftParams] = None, n_sequences: int = 1):
        self.params = params or default_params()
        h = C.c_void_p()
        _check(lib().sssd_draft_create(C.byref(self.params), n_sequences, C.byref(h)), "sssd_draft_create")
        self.handle = h

    def sssd_draft_input_reset(self, seq: int) -> None:
        _check(lib().sssd_draft_input_reset(self.handle, seq), "sssd_draft_input_reset")

    def sssd_draft_input_append(self, seq: int, tokens: Sequence[int]) -> None:
        t = _i32(tokens)
        _check(lib().sssd_draft_input_append(self.handle, seq, t.ctypes.data, t.size), "sssd_draft_input_append")

    def sssd_draft_datastore_add(self, tokens: Sequence[int]) -> None:
        t = _i32(tokens)
        _check(lib().sssd_draft_datastore_add(self.handle, t.ctypes.data, t.size), "sssd_draft_datastore_add")

    def sssd_draft_propose(self, seq: int, dec_len: int) -> Tuple[List[int], List[int]]:
        tok = np.zeros(dec_len, dtype=np.int32)
        par = np.zeros(dec_len, dtype=np.int32)
        n = C.c_int32()
        _check(lib().sssd_draft_propose(self.handle, seq, dec_len, tok.ctypes.data, par.ctypes.data, C.byref(n)),
               "sssd_draft_propose")
        return tok[: n.value].tolist(), par[: n.value].tolist()

    def sssd_draft_input_count(self, seq: int, gram: Sequence[int]) -> int:
        g = _i32(gram)
        return int(lib().sssd_draft_input_count(self.handle, seq, g.ctypes.data, g.size))

    def sssd_draft_match_input(self, seq: int) -> List[int]:
        out = np.zeros(self.params.prefix_len, dtype=np.int32)
        n = lib().sssd_draft_match_input(self.handle, seq, out.ctypes.data)
        _check(min(n, 0), "sssd_draft_match_input")
        return out[:n].tolist()

    def sssd_draft_datastore_lookup(self, sub: int, prefix: Sequence[int], max_out: int = 1 << 20) -> Tuple[List[int], int]:
        g = _i32(prefix)
        pos = np.zeros(max_out, dtype=np.int64)
        total = C.c_int64()
        _check(lib().sssd_draft_datastore_lookup(self.handle, sub, g.ctypes.data, g.size, pos.ctypes.data, max_out,
                                                 C.byref(total)), "sssd_draft_datastore_lookup")
        return pos[: min(total.value, max_out)].tolist(), int(total.value)

    def sssd_draft_datastore_tree(self, seq: int):
        cap = 1 + 2 * self.params.prefix_len * self.params.max_samples * self.params.branch_len
        tok = np.zeros(cap, dtype=np.int32)
        par = np.zeros(cap, dtype=np.int32)
        cnt = np.zeros(cap, dtype=np.int64)
        n = C.c_int32()
        _check(lib().sssd_draft_datastore_tree(self.handle, seq, tok.ctypes.data, par.ctypes.data, cnt.ctypes.data,
                                               C.byref(n)), "sssd_draft_datastore_tree")
        return tok[: n.value].tolist(), par[: n.value].tolist(), cnt[: n.value].tolist()

    def sssd_draft_destroy(self) -> None:
        if self.handle:
            _check(lib().sssd_draft_destroy(self.handle), "sssd_draft_destroy")
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.sssd_draft_destroy()
        except Exception:
            pass
