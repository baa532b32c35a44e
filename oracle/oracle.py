"""ctypes front end of the C oracle (wg_oracle.c).  TEST INFRASTRUCTURE ONLY.

Builds the shared object with gcc when it is missing or older than its source.
No part of the HIP library is imported or called from here.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "wg_oracle.c")
_LIB = os.path.join(_DIR, "libwg_oracle.so")
# The test that plants mistakes in copies of the source points this at such a copy, to see the
# pins fail on it; the object is then built next to the copy.
if os.environ.get("WG_ORACLE_SOURCE"):
    _SRC = os.path.abspath(os.environ["WG_ORACLE_SOURCE"])
    _LIB = os.path.join(os.path.dirname(_SRC), "libwg_oracle_planted.so")

SID_FINAL = 0
SID_ERROR = 0xFFFFFFFF
EOS = 256
FLAG_EOS_RESTART = 1
KINDS = {0: "FINAL", 1: "LIT", 2: "WAIT", 3: "COND", 4: "END"}


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _Args(C.Structure):
    _fields_ = [("n", C.c_uint32), ("names", C.POINTER(C.c_char_p)),
                ("data", C.POINTER(C.POINTER(C.c_uint8))), ("lens", C.POINTER(C.c_uint64))]


class _Vocab(C.Structure):
    _fields_ = [("bytes", C.c_void_p), ("offsets", C.c_void_p), ("V", C.c_uint32),
                ("eos_id", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.wgo_compile.restype = C.c_void_p
        L.wgo_compile.argtypes = [C.POINTER(C.c_char_p), C.POINTER(_Args), C.c_uint32, C.c_uint32,
                                  C.c_char_p, C.c_uint64]
        L.wgo_destroy.argtypes = [C.c_void_p]
        for f in ("wgo_num_states",):
            getattr(L, f).restype = C.c_uint32
            getattr(L, f).argtypes = [C.c_void_p]
        for f in ("wgo_start_state", "wgo_end_state"):
            getattr(L, f).restype = C.c_uint32
            getattr(L, f).argtypes = [C.c_void_p, C.c_uint32]
        L.wgo_describe.argtypes = [C.c_void_p, C.c_uint32, C.POINTER(C.c_int64)]
        L.wgo_step.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_int,
                               C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.wgo_walk_token.argtypes = [C.c_void_p, C.POINTER(_Vocab), C.c_uint32, C.c_uint32,
                                     C.c_int64, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.wgo_mask_row.argtypes = [C.c_void_p, C.POINTER(_Vocab), C.c_uint32, C.c_uint32, C.c_void_p]
        L.wgo_fill_masks.argtypes = [C.c_void_p, C.POINTER(_Vocab), C.c_void_p, C.c_uint32, C.c_void_p]
        L.wgo_apply_mask.argtypes = [C.c_void_p, C.c_int, C.c_uint32, C.c_uint32, C.c_int64, C.c_void_p]
        L.wgo_masked_argmax.argtypes = [C.c_void_p, C.c_int, C.c_uint32, C.c_uint32, C.c_int64, C.c_void_p, C.c_void_p]
        L.wgo_masked_topk.argtypes = [C.c_void_p, C.c_int, C.c_uint32, C.c_uint32, C.c_int64, C.c_void_p,
                                      C.c_uint32, C.c_void_p, C.c_void_p]
        L.wgo_advance.argtypes = [C.c_void_p, C.POINTER(_Vocab), C.c_void_p, C.c_void_p, C.c_uint32]
        L.wgo_key_rem.restype = C.c_uint32
        L.wgo_key_rem.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32]
        L.wgo_forced_bytes.restype = C.c_uint32
        L.wgo_forced_bytes.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32)]
        L.wgo_select_bit.restype = C.c_int64
        L.wgo_select_bit.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64]
        L.wgo_trajectory.restype = C.c_int64
        L.wgo_trajectory.argtypes = [C.c_void_p, C.POINTER(_Vocab), C.c_uint32, C.c_void_p,
                                     C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


class OracleVocab:
    def __init__(self, token_bytes, offsets, eos_id):
        self.bytes = np.ascontiguousarray(token_bytes, dtype=np.uint8)
        self.offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
        self.V = len(self.offsets) - 1
        self.eos_id = int(eos_id)
        self.W = (self.V + 31) // 32
        self.lmax = int(np.diff(self.offsets.astype(np.int64)).max()) if self.V else 0
        self.c = _Vocab(self.bytes.ctypes.data, self.offsets.ctypes.data, self.V, self.eos_id)


class Oracle:
    """A compiled set of template instances plus the vocabulary they are run against."""

    def __init__(self, texts, args=None, vocab=None, restart=False):
        L = lib()
        n = len(texts)
        enc = [t.encode("utf-8") if isinstance(t, str) else bytes(t) for t in texts]
        c_texts = (C.c_char_p * max(n, 1))(*enc)
        keep = [enc]
        c_args = None
        if args is not None:
            assert len(args) == n
            c_args = (_Args * max(n, 1))()
            for i, a in enumerate(args):
                names = [k.encode() for k in a]
                vals = [np.frombuffer(bytes(v), dtype=np.uint8).copy() for v in a.values()]
                m = len(names)
                c_names = (C.c_char_p * max(m, 1))(*names)
                c_data = (C.POINTER(C.c_uint8) * max(m, 1))(
                    *[v.ctypes.data_as(C.POINTER(C.c_uint8)) for v in vals])
                c_lens = (C.c_uint64 * max(m, 1))(*[len(v) for v in vals])
                c_args[i] = _Args(m, c_names, c_data, c_lens)
                keep += [names, vals, c_names, c_data, c_lens]
        err = C.create_string_buffer(512)
        self.h = L.wgo_compile(c_texts, c_args, n, FLAG_EOS_RESTART if restart else 0, err, 512)
        if not self.h:
            raise OracleError(err.value.decode(errors="replace"))
        self.n_templates = n
        self.vocab = vocab
        self.num_states = L.wgo_num_states(self.h)

    def __del__(self):
        # at interpreter shutdown the module's globals may already be gone: then the process
        # ends anyway and the handle is left to it
        if getattr(self, "h", None) and lib is not None:
            lib().wgo_destroy(self.h)
            self.h = None

    def start_state(self, t=0):
        return lib().wgo_start_state(self.h, t)

    def end_state(self, t=0):
        return lib().wgo_end_state(self.h, t)

    def describe(self, sid):
        out = (C.c_int64 * 7)()
        if lib().wgo_describe(self.h, sid, out) != 0:
            raise IndexError(sid)
        return {"kind": KINDS[out[0]], "byte": out[1], "max": out[2], "next": out[3],
                "tnext": out[4], "fnext": out[5], "tmpl": out[6]}

    def step(self, sid, aux, symbol):
        """(sid', aux') or None when the symbol is rejected."""
        s, a = C.c_uint32(), C.c_uint32()
        ok = lib().wgo_step(self.h, sid, aux, symbol, C.byref(s), C.byref(a))
        return (s.value, a.value) if ok else None

    def walk_bytes(self, state, data):
        for x in data:
            state = self.step(state[0], state[1], x)
            if state is None:
                return None
        return state

    def walk_token(self, state, t):
        s, a = C.c_uint32(), C.c_uint32()
        ok = lib().wgo_walk_token(self.h, C.byref(self.vocab.c), state[0], state[1], t,
                                  C.byref(s), C.byref(a))
        return (s.value, a.value) if ok else None

    def mask_row(self, state):
        row = np.zeros(self.vocab.W, dtype=np.uint32)
        lib().wgo_mask_row(self.h, C.byref(self.vocab.c), state[0], state[1], row.ctypes.data)
        return row

    def fill_masks(self, states):
        st = np.ascontiguousarray(states, dtype=np.uint32).reshape(-1, 2)
        out = np.zeros((len(st), self.vocab.W), dtype=np.uint32)
        lib().wgo_fill_masks(self.h, C.byref(self.vocab.c), st.ctypes.data, len(st), out.ctypes.data)
        return out

    def advance(self, states, tokens):
        st = np.ascontiguousarray(states, dtype=np.uint32).reshape(-1, 2).copy()
        tk = np.ascontiguousarray(tokens, dtype=np.int32)
        assert len(tk) == len(st)
        lib().wgo_advance(self.h, C.byref(self.vocab.c), st.ctypes.data, tk.ctypes.data, len(st))
        return st

    def forced_bytes(self, sid, cap=64):
        """(bytes, state after them): what a request in `sid` can only produce next (the rest of
        its Write run), at most cap bytes."""
        buf = (C.c_uint8 * max(cap, 1))()
        end = C.c_uint32()
        n = lib().wgo_forced_bytes(self.h, sid, buf, cap, C.byref(end))
        return bytes(buf[:n]), end.value

    def key_rem(self, state, lmax=None):
        return lib().wgo_key_rem(self.h, state[0], state[1],
                                 self.vocab.lmax if lmax is None else lmax)

    def trajectory(self, states, draws):
        """draws uint64 [steps, B] -> (tokens int32 [steps, B], states uint32 [steps, B, 2], n_masks)."""
        st = np.ascontiguousarray(states, dtype=np.uint32).reshape(-1, 2).copy()
        dr = np.ascontiguousarray(draws, dtype=np.uint64)
        steps, B = dr.shape
        assert B == len(st)
        toks = np.zeros((steps, B), dtype=np.int32)
        sts = np.zeros((steps, B, 2), dtype=np.uint32)
        n = lib().wgo_trajectory(self.h, C.byref(self.vocab.c), self.vocab.lmax, st.ctypes.data,
                                 B, steps, dr.ctypes.data, toks.ctypes.data, sts.ctypes.data)
        if n < 0:
            raise MemoryError("oracle trajectory")
        return toks, sts, int(n)


def apply_mask(logits, bitmask, row_stride=None):
    """In-place on a numpy array: float32, or uint16 holding bfloat16 bit patterns."""
    assert logits.flags["C_CONTIGUOUS"] and logits.ndim == 2
    B, cols = logits.shape
    bm = np.ascontiguousarray(bitmask, dtype=np.uint32)
    V = cols if row_stride is None else row_stride[0]
    stride = cols
    if logits.dtype == np.float32:
        dt = 0
    elif logits.dtype == np.uint16:
        dt = 1
    else:
        raise TypeError(logits.dtype)
    assert bm.shape == (B, (V + 31) // 32)
    lib().wgo_apply_mask(logits.ctypes.data, dt, B, V, stride, bm.ctypes.data)
    return logits


def masked_argmax(logits, bitmask):
    """int32 [B]: greedy token per row of a float32 array or a uint16 array of bfloat16 bits."""
    assert logits.flags["C_CONTIGUOUS"] and logits.ndim == 2
    B, V = logits.shape
    bm = np.ascontiguousarray(bitmask, dtype=np.uint32)
    assert bm.shape == (B, (V + 31) // 32)
    dt = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1}[logits.dtype]
    out = np.zeros(B, dtype=np.int32)
    lib().wgo_masked_argmax(logits.ctypes.data, dt, B, V, V, bm.ctypes.data, out.ctypes.data)
    return out


def masked_topk(logits, bitmask, k):
    """(int32 [B, k] token ids, [B, k] raw values of the logits' type): the k best allowed tokens
    per row of a float32 array or a uint16 array of bfloat16 bits, best first; -1 / -inf when
    a row allows fewer than k."""
    assert logits.flags["C_CONTIGUOUS"] and logits.ndim == 2
    B, V = logits.shape
    bm = np.ascontiguousarray(bitmask, dtype=np.uint32)
    assert bm.shape == (B, (V + 31) // 32)
    dt = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1}[logits.dtype]
    ids = np.zeros((B, k), dtype=np.int32)
    vals = np.zeros((B, k), dtype=logits.dtype)
    lib().wgo_masked_topk(logits.ctypes.data, dt, B, V, V, bm.ctypes.data, int(k), ids.ctypes.data, vals.ctypes.data)
    return ids, vals


def select_bit(row, k):
    row = np.ascontiguousarray(row, dtype=np.uint32)
    return int(lib().wgo_select_bit(row.ctypes.data, len(row), int(k)))
