"""ctypes binding of libfsmidx (see ``include/fsmidx.h``).  Argument marshalling only.

Every step of index construction and masking runs in the HIP kernels of the shared library;
this module converts numpy arrays / torch tensors to pointers and sizes and raises
``FsmidxError`` when a call reports a failure.  There is no CPU fallback: if the library has not
been built, loading it raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_int32, c_int64, c_size_t, c_void_p

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfsmidx.so")

OK, INVALID_ARG, OUT_OF_MEMORY, HIP_ERROR, UNSUPPORTED, BAD_DEVICE_INPUT, WORKSPACE_TOO_SMALL = 0, -1, -2, -3, -4, -5, -6
OUTPUT_TOO_SMALL = -7
DTYPE_F32, DTYPE_BF16 = 0, 1

EXPORTS = ("fsmidx_last_error", "fsmidx_validate_host", "fsmidx_build_index", "fsmidx_index_csr",
           "fsmidx_index_to_host", "fsmidx_free_index", "fsmidx_build_workspace_bytes",
           "fsmidx_build_count", "fsmidx_build_fill", "fsmidx_build_into", "fsmidx_build_enqueue", "fsmidx_build_finish", "fsmidx_build_allow_bits", "fsmidx_mask_logits",
           "fsmidx_advance_states", "fsmidx_masked_argmax_workspace_bytes", "fsmidx_masked_argmax", "fsmidx_masked_argmax_static",
           "fsmidx_masked_sample_workspace_bytes", "fsmidx_masked_sample",
           "fsmidx_union_workspace_bytes", "fsmidx_union_dfa",
           "fsmidx_dedupe_workspace_bytes", "fsmidx_dedupe_rows", "fsmidx_dedupe_fill",
           "fsmidx_minimise_workspace_bytes", "fsmidx_minimise_dfa",
           "fsmidx_reach_workspace_bytes", "fsmidx_reachable_states", "fsmidx_restrict_rows", "fsmidx_restrict_fill",
           "fsmidx_scanner_workspace_bytes", "fsmidx_scanner_terminal_sets", "fsmidx_scanner_restart_table",
           "fsmidx_profile_enable", "fsmidx_profile_read")


class FsmidxError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"fsmidx error {code}: {message}")
        self.code = code


class OutputTooSmall(FsmidxError):
    """fsmidx_build_into found more entries than the caller's arrays hold; ``nnz`` says how many."""

    def __init__(self, message: str):
        super().__init__(OUTPUT_TOO_SMALL, message)
        self.nnz = -1


class CDfa(Structure):
    _fields_ = [("trans", c_void_p), ("n_states", c_int32), ("n_classes", c_int32),
                ("byte_to_class", c_void_p), ("accept", c_void_p), ("dead_state", c_int32)]


class CVocab(Structure):
    _fields_ = [("bytes", c_void_p), ("offsets", c_void_p), ("n_tokens", c_int32),
                ("eos_token_id", c_int32), ("n_bytes", c_int64)]


class CCsr(Structure):
    _fields_ = [("n_states", c_int32), ("n_tokens", c_int32), ("nnz", c_int64),
                ("row_ptr", c_void_p), ("token_ids", c_void_p), ("next_states", c_void_p),
                ("allow_bits", c_void_p), ("allow_stride", c_int64)]


_lib = None


def load():
    """Load libfsmidx.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2307_09702_amd.build` "
                           "(hipcc, --offload-arch=gfx950); there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    lib.fsmidx_last_error.restype = c_char_p
    lib.fsmidx_last_error.argtypes = []
    lib.fsmidx_validate_host.argtypes = [POINTER(CDfa), POINTER(CVocab)]
    lib.fsmidx_build_index.argtypes = [POINTER(CDfa), POINTER(CVocab), c_void_p, POINTER(c_void_p)]
    lib.fsmidx_index_csr.argtypes = [c_void_p, POINTER(CCsr)]
    lib.fsmidx_index_to_host.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    lib.fsmidx_free_index.argtypes = [c_void_p]
    lib.fsmidx_free_index.restype = None
    lib.fsmidx_build_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int64, POINTER(c_size_t)]
    lib.fsmidx_build_count.argtypes = [POINTER(CDfa), POINTER(CVocab), c_void_p, c_size_t, c_void_p,
                                       POINTER(c_int64), c_void_p]
    lib.fsmidx_build_fill.argtypes = [POINTER(CDfa), POINTER(CVocab), c_void_p, c_size_t, c_void_p, c_int64,
                                      c_void_p, c_void_p, c_void_p]
    lib.fsmidx_build_into.argtypes = [POINTER(CDfa), POINTER(CVocab), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p,
                                      c_int64, POINTER(c_int64), c_void_p]
    lib.fsmidx_build_enqueue.argtypes = [POINTER(CDfa), POINTER(CVocab), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p,
                                         c_int64, c_void_p]
    lib.fsmidx_build_finish.argtypes = [POINTER(CDfa), POINTER(CVocab), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p,
                                        c_int64, POINTER(c_int64), POINTER(c_int32), c_void_p]
    lib.fsmidx_build_allow_bits.argtypes = [c_int32, c_int32, c_int32, c_int64, c_void_p, POINTER(c_void_p),
                                            POINTER(c_int64)]
    lib.fsmidx_mask_logits.argtypes = [POINTER(CCsr), c_void_p, c_int32, c_void_p, c_void_p, c_int64, c_int32,
                                       c_void_p]
    lib.fsmidx_advance_states.argtypes = [POINTER(CCsr), c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
    lib.fsmidx_masked_argmax_workspace_bytes.argtypes = [c_int32, POINTER(c_size_t)]
    lib.fsmidx_masked_argmax.argtypes = [POINTER(CCsr), c_void_p, c_int32, c_void_p, c_int64, c_int32, c_void_p,
                                         c_size_t, c_void_p, c_void_p, c_void_p]
    lib.fsmidx_masked_argmax_static.argtypes = [POINTER(CCsr), c_void_p, c_int32, c_void_p, c_int64, c_int32, c_void_p,
                                                c_void_p, c_void_p]
    lib.fsmidx_masked_sample_workspace_bytes.argtypes = [c_int32, POINTER(c_size_t)]
    lib.fsmidx_masked_sample.argtypes = [POINTER(CCsr), c_void_p, c_int32, c_void_p, c_int64, c_int32, c_void_p,
                                         c_void_p, c_size_t, c_void_p, c_void_p, c_void_p]
    lib.fsmidx_union_workspace_bytes.argtypes = [c_int32, POINTER(c_size_t)]
    lib.fsmidx_union_dfa.argtypes = [POINTER(CDfa), c_int32, c_void_p, c_int64, c_void_p, c_void_p, c_void_p, c_size_t,
                                     POINTER(CDfa), POINTER(c_int32), c_void_p]
    lib.fsmidx_dedupe_workspace_bytes.argtypes = [c_int32, POINTER(c_size_t)]
    lib.fsmidx_dedupe_rows.argtypes = [POINTER(CCsr), c_void_p, c_size_t, c_void_p, c_void_p, POINTER(c_int32),
                                       POINTER(c_int64), c_void_p]
    lib.fsmidx_dedupe_fill.argtypes = [POINTER(CCsr), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.fsmidx_minimise_workspace_bytes.argtypes = [c_int32, POINTER(c_size_t)]
    lib.fsmidx_minimise_dfa.argtypes = [POINTER(CDfa), c_void_p, c_size_t, c_void_p, c_void_p, c_int64, c_void_p,
                                        POINTER(CDfa), c_void_p]
    lib.fsmidx_reach_workspace_bytes.argtypes = [c_int32, POINTER(c_size_t)]
    lib.fsmidx_reachable_states.argtypes = [POINTER(CCsr), POINTER(c_int32), c_int32, c_void_p, c_size_t, c_void_p,
                                            POINTER(c_int32), c_void_p]
    lib.fsmidx_restrict_rows.argtypes = [POINTER(CCsr), c_void_p, c_void_p, c_size_t, c_void_p, POINTER(c_int64), c_void_p]
    lib.fsmidx_restrict_fill.argtypes = [POINTER(CCsr), c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_void_p]
    lib.fsmidx_scanner_workspace_bytes.argtypes = [c_int32, c_int32, POINTER(c_size_t)]
    lib.fsmidx_scanner_terminal_sets.argtypes = [POINTER(CDfa), c_void_p, c_void_p, c_size_t, c_void_p, POINTER(c_int32),
                                                 c_void_p]
    lib.fsmidx_scanner_restart_table.argtypes = [POINTER(CDfa), c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p,
                                                 c_size_t, c_void_p, c_void_p]
    lib.fsmidx_profile_enable.argtypes = [ctypes.c_int]
    lib.fsmidx_profile_read.argtypes = [POINTER(ctypes.c_double), POINTER(c_int64)]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.argtypes is None:
            # (without them ctypes passes a Python int as a 32-bit int: a device address would be cut in half)
            raise RuntimeError(f"binding.load: {name} has no argument types")
        if name not in ("fsmidx_last_error", "fsmidx_free_index"):
            fn.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != OK:
        raise FsmidxError(rc, load().fsmidx_last_error().decode(errors="replace"))


def _ptr(x) -> int | None:
    """Address of a numpy array or a torch tensor (None stays NULL)."""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream_handle(stream) -> int | None:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _structs(trans, byte_to_class, accept, dead_state, vocab_bytes, offsets, eos_token_id, n_bytes=None):
    n_states, n_classes = int(trans.shape[0]), int(trans.shape[1])
    n_tokens = int(offsets.shape[0]) - 1
    if n_bytes is None:
        n_bytes = int(vocab_bytes.shape[0]) if vocab_bytes is not None else 0
    d = CDfa(_ptr(trans), n_states, n_classes, _ptr(byte_to_class), _ptr(accept), int(dead_state))
    v = CVocab(_ptr(vocab_bytes) if n_bytes else None, _ptr(offsets), n_tokens, int(eos_token_id), int(n_bytes))
    return d, v


def _host_arrays(trans, byte_to_class, accept, vocab_bytes, offsets):
    trans = np.ascontiguousarray(trans, dtype=np.int32)
    if trans.ndim != 2:
        raise ValueError("trans must be [n_states, n_classes]")
    return (trans, np.ascontiguousarray(byte_to_class, dtype=np.uint8), np.ascontiguousarray(accept, dtype=np.uint8),
            np.ascontiguousarray(vocab_bytes, dtype=np.uint8), np.ascontiguousarray(offsets, dtype=np.int64))


def validate_host(trans, byte_to_class, accept, dead_state, vocab_bytes, offsets, eos_token_id=-1, n_bytes=None):
    """fsmidx_validate_host on numpy inputs; raises FsmidxError(INVALID_ARG) on malformed input."""
    arrs = _host_arrays(trans, byte_to_class, accept, vocab_bytes, offsets)
    d, v = _structs(arrs[0], arrs[1], arrs[2], dead_state, arrs[3], arrs[4], eos_token_id, n_bytes)
    _check(load().fsmidx_validate_host(byref(d), byref(v)))


class IndexHandle:
    """Owner of a CSR index in device memory (fsmidx_index*)."""

    def __init__(self, handle: int):
        self._h = handle
        self.csr = CCsr()
        _check(load().fsmidx_index_csr(self._h, byref(self.csr)))

    @property
    def nnz(self) -> int:
        return int(self.csr.nnz)

    def to_host(self):
        n_states, nnz = int(self.csr.n_states), int(self.csr.nnz)
        row_ptr = np.empty(n_states + 1, np.int64)
        token_ids = np.empty(nnz, np.int32)
        next_states = np.empty(nnz, np.int32)
        _check(load().fsmidx_index_to_host(self._h, _ptr(row_ptr), _ptr(token_ids) if nnz else None,
                                           _ptr(next_states) if nnz else None))
        return row_ptr, token_ids, next_states

    def free(self):
        if self._h:
            load().fsmidx_free_index(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def build_index(trans, byte_to_class, accept, dead_state, vocab_bytes, offsets, eos_token_id=-1, stream=None,
                n_bytes=None) -> IndexHandle:
    """fsmidx_build_index: host numpy inputs -> index owned by the library."""
    arrs = _host_arrays(trans, byte_to_class, accept, vocab_bytes, offsets)
    d, v = _structs(arrs[0], arrs[1], arrs[2], dead_state, arrs[3], arrs[4], eos_token_id, n_bytes)
    out = c_void_p()
    _check(load().fsmidx_build_index(byref(d), byref(v), _stream_handle(stream), byref(out)))
    return IndexHandle(out.value)


def build_workspace_bytes(n_states: int, n_classes: int, n_tokens: int, n_bytes: int) -> int:
    size = c_size_t()
    _check(load().fsmidx_build_workspace_bytes(n_states, n_classes, n_tokens, n_bytes, byref(size)))
    return int(size.value)


def _aligned(n_bytes: int, device):
    """(tensor that owns the memory, 256-byte aligned address inside it)"""
    import torch
    buf = torch.empty(n_bytes + 256, dtype=torch.uint8, device=device)
    return buf, (buf.data_ptr() + 255) & ~255


class DeviceUnion:
    """fsmidx_union_dfa: automata given as numpy (trans, byte_to_class, accept, dead) tuples are put
    on the device and joined there into one automaton (device tensors ``trans``, ``byte_to_class``,
    ``accept``; ``n_states``, ``n_classes``, ``dead_state``; ``state_base`` as a numpy array)."""

    def __init__(self, automata, device="cuda:0", trans_capacity=None, stream=None):
        import torch
        self.device = torch.device(device)
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.device)
        self.parts = []
        structs = (CDfa * len(automata))()
        total = 0
        for k, (trans, b2c, accept, dead) in enumerate(automata):
            t = to(np.asarray(trans, dtype=np.int32)); b = to(np.asarray(b2c, dtype=np.uint8))
            a = to(np.asarray(accept, dtype=np.uint8))
            self.parts.append((t, b, a))
            structs[k] = CDfa(t.data_ptr(), int(trans.shape[0]), int(trans.shape[1]), b.data_ptr(), a.data_ptr(), int(dead))
            total += int(trans.shape[0])
        if trans_capacity is None:
            trans_capacity = total * 256
        self.trans_full = torch.empty(max(trans_capacity, 1), dtype=torch.int32, device=self.device)
        self.byte_to_class = torch.empty(256, dtype=torch.uint8, device=self.device)
        self.accept = torch.empty(max(total, 1), dtype=torch.uint8, device=self.device)
        need = c_size_t()
        _check(load().fsmidx_union_workspace_bytes(len(automata), byref(need)))
        self._ws, ws_ptr = _aligned(int(need.value), self.device)
        out = CDfa()
        base = (c_int32 * (len(automata) + 1))()
        _check(load().fsmidx_union_dfa(structs, len(automata), self.trans_full.data_ptr(), int(trans_capacity),
                                       self.byte_to_class.data_ptr(), self.accept.data_ptr(), ws_ptr, int(need.value),
                                       byref(out), base, _stream_handle(stream)))
        self.n_states, self.n_classes, self.dead_state = int(out.n_states), int(out.n_classes), int(out.dead_state)
        self.trans = self.trans_full[:self.n_states * self.n_classes].view(self.n_states, self.n_classes)
        self.state_base = np.array(list(base), dtype=np.int64)


class DeviceMinimised:
    """fsmidx_minimise_dfa: an automaton given as numpy arrays (or device tensors) is put on the
    device and reduced there (device tensors ``trans`` [classes x n_classes], ``byte_to_class``,
    ``accept``, ``block_of_state`` [states of the input]; ``n_states`` = number of classes)."""

    def __init__(self, trans, byte_to_class, accept, dead_state, device="cuda:0", trans_capacity=None, stream=None):
        import torch
        self.device = torch.device(device)
        to = lambda a, dt: a if hasattr(a, "data_ptr") and not isinstance(a, np.ndarray) else \
            torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=dt))).to(self.device)
        self._in = (to(trans, np.int32), to(byte_to_class, np.uint8), to(accept, np.uint8))
        n_states, n_classes = int(self._in[0].shape[0]), int(self._in[0].shape[1])
        if trans_capacity is None:
            trans_capacity = n_states * n_classes
        self.trans_full = torch.empty(max(trans_capacity, 1), dtype=torch.int32, device=self.device)
        self.accept = torch.empty(n_states, dtype=torch.uint8, device=self.device)
        self.block_of_state = torch.empty(n_states, dtype=torch.int32, device=self.device)
        self.byte_to_class = self._in[1]
        need = c_size_t()
        _check(load().fsmidx_minimise_workspace_bytes(n_states, byref(need)))
        ws, ws_ptr = _aligned(int(need.value), self.device)
        src = CDfa(self._in[0].data_ptr(), n_states, n_classes, self._in[1].data_ptr(), self._in[2].data_ptr(), int(dead_state))
        out = CDfa()
        _check(load().fsmidx_minimise_dfa(byref(src), ws_ptr, int(need.value), self.block_of_state.data_ptr(),
                                          self.trans_full.data_ptr(), int(trans_capacity), self.accept.data_ptr(),
                                          byref(out), _stream_handle(stream)))
        del ws
        self.n_states, self.n_classes, self.dead_state = int(out.n_states), int(out.n_classes), int(out.dead_state)
        self.trans = self.trans_full[:self.n_states * self.n_classes].view(self.n_states, self.n_classes)


class DeviceScanner:
    """The scanners of all parse states in one automaton, on the device (fsmidx_scanner_*).
    ``trans`` int32 [Q, C], ``completes`` uint64 [Q], ``scanner_of_state`` int32 [Q], ``shift`` int32
    [n_parse_states, n_terminals]: numpy arrays or device tensors (uint64 as int64 bit patterns)."""

    def __init__(self, trans, dead_state, completes, scanner_of_state, shift, device="cuda:0"):
        import torch
        self.device = torch.device(device)

        def to(a, dt):
            if hasattr(a, "data_ptr") and not isinstance(a, np.ndarray):
                return a
            return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=dt))).to(self.device)
        self.trans = to(trans, np.int32)
        self.completes = to(np.asarray(completes).view(np.int64) if isinstance(completes, np.ndarray) else completes, np.int64)
        self.scanner_of_state = to(scanner_of_state, np.int32)
        self.shift = to(shift, np.int32)
        self.n_states, self.n_classes = int(self.trans.shape[0]), int(self.trans.shape[1])
        self.n_parse_states, self.n_terminals = int(self.shift.shape[0]), int(self.shift.shape[1])
        self.dead_state = int(dead_state)
        need = c_size_t()
        _check(load().fsmidx_scanner_workspace_bytes(self.n_states, self.n_classes, byref(need)))
        self.ws_bytes = int(need.value)
        self._ws, self.ws_ptr = _aligned(self.ws_bytes, self.device)
        self.c_dfa = CDfa(self.trans.data_ptr(), self.n_states, self.n_classes, None, None, self.dead_state)

    def terminal_sets(self, out=None, stream=None):
        """Returns (possible int64 [Q] on the device: the uint64 masks' bit patterns, launches)."""
        import torch
        if out is None:
            out = torch.empty(self.n_states, dtype=torch.int64, device=self.device)
        launches = c_int32()
        _check(load().fsmidx_scanner_terminal_sets(byref(self.c_dfa), self.completes.data_ptr(), self.ws_ptr,
                                                   self.ws_bytes, out.data_ptr(), byref(launches),
                                                   _stream_handle(stream)))
        return out, int(launches.value)

    def restart_table(self, out=None, stream=None):
        """Returns trans_out int32 [Q, C] on the device."""
        import torch
        if out is None:
            out = torch.empty((self.n_states, self.n_classes), dtype=torch.int32, device=self.device)
        _check(load().fsmidx_scanner_restart_table(byref(self.c_dfa), self.completes.data_ptr(),
                                                   self.scanner_of_state.data_ptr(), self.shift.data_ptr(),
                                                   self.n_parse_states, self.n_terminals, self.ws_ptr, self.ws_bytes,
                                                   out.data_ptr(), _stream_handle(stream)))
        return out


def dedupe_rows(csr: CCsr, device="cuda:0", stream=None):
    """fsmidx_dedupe_rows + fsmidx_dedupe_fill on torch tensors.  Returns (row_of_state int32
    [n_states], unique_row_ptr int64 [n_unique + 1], token_ids_u, next_states_u)."""
    import torch
    dev = torch.device(device)
    n_states = int(csr.n_states)
    need = c_size_t()
    _check(load().fsmidx_dedupe_workspace_bytes(n_states, byref(need)))
    ws, ws_ptr = _aligned(int(need.value), dev)
    row_of = torch.empty(n_states, dtype=torch.int32, device=dev)
    urp = torch.empty(n_states + 1, dtype=torch.int64, device=dev)
    n_unique, nnz_unique = c_int32(), c_int64()
    _check(load().fsmidx_dedupe_rows(byref(csr), ws_ptr, int(need.value), row_of.data_ptr(), urp.data_ptr(),
                                     byref(n_unique), byref(nnz_unique), _stream_handle(stream)))
    tok = torch.empty(max(int(nnz_unique.value), 1), dtype=torch.int32, device=dev)
    nxt = torch.empty(max(int(nnz_unique.value), 1), dtype=torch.int32, device=dev)
    _check(load().fsmidx_dedupe_fill(byref(csr), ws_ptr, int(need.value), urp.data_ptr(), tok.data_ptr(), nxt.data_ptr(),
                                     _stream_handle(stream)))
    torch.cuda.synchronize()
    del ws
    return row_of, urp[:int(n_unique.value) + 1], tok[:int(nnz_unique.value)], nxt[:int(nnz_unique.value)]


def reachable_states(csr: CCsr, starts, device="cuda:0", stream=None):
    """fsmidx_reachable_states on torch tensors.  Returns (reach uint8 [n_states] on the device,
    number of reachable states)."""
    import torch
    dev = torch.device(device)
    n_states = int(csr.n_states)
    need = c_size_t()
    _check(load().fsmidx_reach_workspace_bytes(n_states, byref(need)))
    ws, ws_ptr = _aligned(int(need.value), dev)
    reach = torch.empty(n_states, dtype=torch.uint8, device=dev)
    starts = [int(s) for s in starts]
    arr = (c_int32 * max(len(starts), 1))(*starts)
    n_reached = c_int32()
    _check(load().fsmidx_reachable_states(byref(csr), arr, len(starts), ws_ptr, int(need.value), reach.data_ptr(),
                                          byref(n_reached), _stream_handle(stream)))
    del ws
    return reach, int(n_reached.value)


def restrict_rows(csr: CCsr, keep, device="cuda:0", stream=None):
    """fsmidx_restrict_rows + fsmidx_restrict_fill on torch tensors (``keep``: uint8 [n_states] on
    the device).  Returns (row_ptr int64 [n_states + 1], token_ids, next_states)."""
    import torch
    dev = torch.device(device)
    n_states = int(csr.n_states)
    need = c_size_t()
    _check(load().fsmidx_reach_workspace_bytes(n_states, byref(need)))
    ws, ws_ptr = _aligned(int(need.value), dev)
    row_ptr = torch.empty(n_states + 1, dtype=torch.int64, device=dev)
    nnz = c_int64()
    _check(load().fsmidx_restrict_rows(byref(csr), keep.data_ptr(), ws_ptr, int(need.value), row_ptr.data_ptr(),
                                       byref(nnz), _stream_handle(stream)))
    tok = torch.empty(max(int(nnz.value), 1), dtype=torch.int32, device=dev)
    nxt = torch.empty(max(int(nnz.value), 1), dtype=torch.int32, device=dev)
    _check(load().fsmidx_restrict_fill(byref(csr), keep.data_ptr(), row_ptr.data_ptr(), tok.data_ptr(), nxt.data_ptr(),
                                       int(nnz.value), _stream_handle(stream)))
    torch.cuda.synchronize()
    del ws
    return row_ptr, tok[:int(nnz.value)], nxt[:int(nnz.value)]


class DeviceProblem:
    """An automaton and a vocabulary resident in device memory (torch tensors own the bytes).
    ``trans``, ``byte_to_class`` and ``accept`` may also be torch tensors already on the device
    (say, the arrays of a DeviceUnion)."""

    def __init__(self, trans, byte_to_class, accept, dead_state, vocab_bytes, offsets, eos_token_id=-1,
                 device="cuda:0"):
        import torch
        if not isinstance(trans, np.ndarray) and hasattr(trans, "data_ptr"):
            self._init_from_device(trans, byte_to_class, accept, dead_state, vocab_bytes, offsets, eos_token_id, device)
            return
        arrs = _host_arrays(trans, byte_to_class, accept, vocab_bytes, offsets)
        self.n_states, self.n_classes = arrs[0].shape
        self.n_tokens = arrs[4].shape[0] - 1
        self.n_bytes = int(arrs[3].shape[0])
        self.dead_state, self.eos_token_id = int(dead_state), int(eos_token_id)
        self.device = torch.device(device)
        to = lambda a: torch.from_numpy(a if a.size else np.zeros(1, a.dtype)).to(self.device)
        self.trans, self.byte_to_class, self.accept, self.vocab_bytes, self.offsets = map(to, arrs)
        self.workspace_bytes = build_workspace_bytes(self.n_states, self.n_classes, self.n_tokens, self.n_bytes)
        self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
        self._ws_ptr = (self.workspace.data_ptr() + 255) & ~255
        self.row_ptr = torch.empty(self.n_states + 1, dtype=torch.int64, device=self.device)
        self.dfa_struct, self.vocab_struct = _structs(self.trans, self.byte_to_class, self.accept, self.dead_state,
                                                      self.vocab_bytes, self.offsets, self.eos_token_id, self.n_bytes)

    def _init_from_device(self, trans, byte_to_class, accept, dead_state, vocab_bytes, offsets, eos_token_id, device):
        import torch
        self.device = torch.device(device)
        self.n_states, self.n_classes = int(trans.shape[0]), int(trans.shape[1])
        vb = np.ascontiguousarray(vocab_bytes, dtype=np.uint8)
        off = np.ascontiguousarray(offsets, dtype=np.int64)
        self.n_tokens, self.n_bytes = off.shape[0] - 1, int(vb.shape[0])
        self.dead_state, self.eos_token_id = int(dead_state), int(eos_token_id)
        self.trans, self.byte_to_class, self.accept = trans.contiguous(), byte_to_class, accept
        to = lambda a: torch.from_numpy(a if a.size else np.zeros(1, a.dtype)).to(self.device)
        self.vocab_bytes, self.offsets = to(vb), to(off)
        self.workspace_bytes = build_workspace_bytes(self.n_states, self.n_classes, self.n_tokens, self.n_bytes)
        self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
        self._ws_ptr = (self.workspace.data_ptr() + 255) & ~255
        self.row_ptr = torch.empty(self.n_states + 1, dtype=torch.int64, device=self.device)
        self.dfa_struct, self.vocab_struct = _structs(self.trans, self.byte_to_class, self.accept, self.dead_state,
                                                      self.vocab_bytes, self.offsets, self.eos_token_id, self.n_bytes)

    def count(self, stream=None) -> int:
        """fsmidx_build_count: fills ``row_ptr`` and returns nnz."""
        nnz = c_int64()
        _check(load().fsmidx_build_count(byref(self.dfa_struct), byref(self.vocab_struct), self._ws_ptr,
                                         self.workspace_bytes, self.row_ptr.data_ptr(), byref(nnz),
                                         _stream_handle(stream)))
        return int(nnz.value)

    def fill(self, nnz: int, token_ids, next_states, stream=None):
        """fsmidx_build_fill into caller tensors of at least ``nnz`` int32 each."""
        _check(load().fsmidx_build_fill(byref(self.dfa_struct), byref(self.vocab_struct), self._ws_ptr,
                                        self.workspace_bytes, self.row_ptr.data_ptr(), nnz,
                                        _ptr(token_ids) if nnz else None, _ptr(next_states) if nnz else None,
                                        _stream_handle(stream)))

    def build_into(self, token_ids, next_states, stream=None) -> int:
        """fsmidx_build_into: the whole build into caller tensors in one call; returns nnz.  Raises
        OutputTooSmall (with ``.nnz``) if the tensors hold fewer entries than the index has."""
        nnz = c_int64()
        capacity = min(token_ids.numel(), next_states.numel())
        rc = load().fsmidx_build_into(byref(self.dfa_struct), byref(self.vocab_struct), self._ws_ptr,
                                      self.workspace_bytes, self.row_ptr.data_ptr(),
                                      _ptr(token_ids) if capacity else None, _ptr(next_states) if capacity else None,
                                      capacity, byref(nnz), _stream_handle(stream))
        if rc == OUTPUT_TOO_SMALL:
            err = OutputTooSmall(load().fsmidx_last_error().decode())
            err.nnz = int(nnz.value)
            raise err
        _check(rc)
        return int(nnz.value)

    def build_enqueue(self, token_ids, next_states, stream=None) -> None:
        """fsmidx_build_enqueue: the launches of build_into, without waiting for them."""
        capacity = min(token_ids.numel(), next_states.numel())
        _check(load().fsmidx_build_enqueue(byref(self.dfa_struct), byref(self.vocab_struct), self._ws_ptr,
                                           self.workspace_bytes, self.row_ptr.data_ptr(),
                                           _ptr(token_ids) if capacity else None, _ptr(next_states) if capacity else None,
                                           capacity, _stream_handle(stream)))

    def build_finish(self, token_ids, next_states, stream=None):
        """fsmidx_build_finish: waits, returns (nnz, redone)."""
        nnz, redone = c_int64(), c_int32()
        capacity = min(token_ids.numel(), next_states.numel())
        rc = load().fsmidx_build_finish(byref(self.dfa_struct), byref(self.vocab_struct), self._ws_ptr,
                                        self.workspace_bytes, self.row_ptr.data_ptr(),
                                        _ptr(token_ids) if capacity else None, _ptr(next_states) if capacity else None,
                                        capacity, byref(nnz), byref(redone), _stream_handle(stream))
        if rc == OUTPUT_TOO_SMALL:
            err = OutputTooSmall(load().fsmidx_last_error().decode())
            err.nnz = int(nnz.value)
            raise err
        _check(rc)
        return int(nnz.value), bool(redone.value)

    def build(self, stream=None):
        """count + allocate + fill; returns (csr struct, token_ids tensor, next_states tensor)."""
        import torch
        nnz = self.count(stream)
        token_ids = torch.empty(max(nnz, 1), dtype=torch.int32, device=self.device)
        next_states = torch.empty(max(nnz, 1), dtype=torch.int32, device=self.device)
        self.fill(nnz, token_ids, next_states, stream)
        return self.csr(nnz, token_ids, next_states), token_ids[:nnz], next_states[:nnz]

    def allow_bits(self):
        """(device address, words per state) of the bitmap form of the index in the workspace."""
        bits, stride = c_void_p(), c_int64()
        _check(load().fsmidx_build_allow_bits(self.n_states, self.n_classes, self.n_tokens, self.n_bytes,
                                              self._ws_ptr, byref(bits), byref(stride)))
        return bits.value, int(stride.value)

    def csr(self, nnz: int, token_ids, next_states=None, with_bits: bool = True) -> CCsr:
        bits, stride = self.allow_bits() if with_bits else (None, 0)
        return CCsr(self.n_states, self.n_tokens, nnz, self.row_ptr.data_ptr(), _ptr(token_ids),
                    _ptr(next_states) if next_states is not None else None, bits, stride)


PROFILE_PHASES = ("prepare", "count_walk", "scan", "emit_walk", "mask_f32", "mask_bf16",
                  "advance_states", "masked_argmax_f32", "masked_argmax_bf16", "masked_sample_f32",
                  "masked_sample_bf16")


def profile_enable(enabled: bool = True):
    _check(load().fsmidx_profile_enable(1 if enabled else 0))


def profile_read() -> dict:
    """{phase: (mean milliseconds, launches)} since profiling was enabled (waits for the GPU)."""
    ms = (ctypes.c_double * len(PROFILE_PHASES))()
    calls = (c_int64 * len(PROFILE_PHASES))()
    _check(load().fsmidx_profile_read(ms, calls))
    return {name: (float(ms[i]), int(calls[i])) for i, name in enumerate(PROFILE_PHASES)}


def mask_logits(csr: CCsr, states, logits_in, logits_out=None, row_stride=None, dtype=None, stream=None):
    """fsmidx_mask_logits on torch tensors: ``states`` int32 [batch], logits [batch, >= n_tokens]
    float32 or bfloat16.  ``logits_out=None`` masks in place."""
    import torch
    if logits_out is None:
        logits_out = logits_in
    if dtype is None:
        dtype = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}.get(logits_in.dtype, -1)
    if row_stride is None:
        row_stride = logits_in.stride(0) if logits_in.dim() == 2 else int(csr.n_tokens)
    _check(load().fsmidx_mask_logits(byref(csr), _ptr(states), int(states.shape[0]), _ptr(logits_in),
                                     _ptr(logits_out), int(row_stride), int(dtype), _stream_handle(stream)))
    return logits_out



def advance_states(csr: CCsr, states, tokens, states_out=None, stream=None):
    """fsmidx_advance_states on torch tensors: ``states`` and ``tokens`` int32 [batch].
    ``states_out=None`` gives a new tensor; passing ``states`` itself updates in place."""
    import torch
    if states_out is None:
        states_out = torch.empty_like(states)
    _check(load().fsmidx_advance_states(byref(csr), _ptr(states), _ptr(tokens), int(states.shape[0]),
                                        _ptr(states_out), _stream_handle(stream)))
    return states_out


def masked_argmax_workspace_bytes(batch: int) -> int:
    n = c_size_t(0)
    _check(load().fsmidx_masked_argmax_workspace_bytes(int(batch), byref(n)))
    return int(n.value)


def masked_argmax(csr: CCsr, states, logits, workspace=None, tokens_out=None, states_out=None,
                  row_stride=None, dtype=None, stream=None):
    """fsmidx_masked_argmax on torch tensors: ``states`` int32 [batch], logits [batch, >= n_tokens]
    float32 or bfloat16.  Returns (tokens, new states), int32 [batch] each.  ``workspace``: a uint8
    tensor of at least masked_argmax_workspace_bytes(batch) bytes (a new one if None)."""
    import torch
    batch = int(states.shape[0])
    if dtype is None:
        dtype = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}.get(logits.dtype, -1)
    if row_stride is None:
        row_stride = logits.stride(0) if logits.dim() == 2 else int(csr.n_tokens)
    if workspace is None:
        workspace = torch.empty(max(masked_argmax_workspace_bytes(batch), 8), dtype=torch.uint8,
                                device=states.device)
    if tokens_out is None:
        tokens_out = torch.empty_like(states)
    if states_out is None:
        states_out = torch.empty_like(states)
    _check(load().fsmidx_masked_argmax(byref(csr), _ptr(states), batch, _ptr(logits), int(row_stride), int(dtype),
                                       _ptr(workspace), int(workspace.numel()), _ptr(tokens_out), _ptr(states_out),
                                       _stream_handle(stream)))
    return tokens_out, states_out


def masked_argmax_static(csr: CCsr, states, logits, tokens_out, states_out, row_stride=None, dtype=None, stream=None):
    """fsmidx_masked_argmax_static: masked_argmax with the library's own fixed scratch array
    (batch <= 4096); the caller passes the output tensors, nothing is allocated."""
    import torch
    batch = int(states.shape[0])
    if dtype is None:
        dtype = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}.get(logits.dtype, -1)
    if row_stride is None:
        row_stride = logits.stride(0) if logits.dim() == 2 else int(csr.n_tokens)
    _check(load().fsmidx_masked_argmax_static(byref(csr), _ptr(states), batch, _ptr(logits), int(row_stride), int(dtype),
                                              _ptr(tokens_out), _ptr(states_out), _stream_handle(stream)))
    return tokens_out, states_out


def masked_sample_workspace_bytes(batch: int) -> int:
    n = c_size_t(0)
    _check(load().fsmidx_masked_sample_workspace_bytes(int(batch), byref(n)))
    return int(n.value)


def masked_sample(csr: CCsr, states, logits, uniforms, workspace=None, tokens_out=None, states_out=None,
                  row_stride=None, dtype=None, stream=None):
    """fsmidx_masked_sample on torch tensors: ``states`` int32 [batch], logits [batch, >= n_tokens]
    float32 or bfloat16, ``uniforms`` float32 [batch] in [0, 1).  Returns (tokens, new states)."""
    import torch
    batch = int(states.shape[0])
    if dtype is None:
        dtype = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}.get(logits.dtype, -1)
    if row_stride is None:
        row_stride = logits.stride(0) if logits.dim() == 2 else int(csr.n_tokens)
    if workspace is None:
        workspace = torch.empty(max(masked_sample_workspace_bytes(batch), 8), dtype=torch.uint8,
                                device=states.device)
    if tokens_out is None:
        tokens_out = torch.empty_like(states)
    if states_out is None:
        states_out = torch.empty_like(states)
    _check(load().fsmidx_masked_sample(byref(csr), _ptr(states), batch, _ptr(logits), int(row_stride), int(dtype),
                                       _ptr(uniforms), _ptr(workspace), int(workspace.numel()), _ptr(tokens_out),
                                       _ptr(states_out), _stream_handle(stream)))
    return tokens_out, states_out

