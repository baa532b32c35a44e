"""ctypes binding of libwgrammar.so: same names as the C ABI, argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams, nothing
else).  There is no fallback: if the shared library is missing, loading fails.
"""
import ctypes as C
import os

import numpy as np
# torch is imported before the shared library is opened on purpose: the process must hold
# exactly one HIP runtime, and it has to be the one torch's device tensors and streams
# belong to.  libwgrammar.so then binds to that already-loaded runtime by its soname.
import torch  # noqa: F401

from . import build as _build

F32, BF16 = 0, 1
EOS_STOP, EOS_RESTART = 0, 1
SHARE_STATES = 2          # or-ed to either: states with equal futures share their cache keys
SID_FINAL, SID_ERROR = 0, 0xFFFFFFFF

_lib = None


class WgError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("wg status %d: %s" % (code, msg))
        self.code = code


class _Args(C.Structure):
    _fields_ = [("n", C.c_uint32), ("names", C.POINTER(C.c_char_p)),
                ("data", C.POINTER(C.POINTER(C.c_uint8))), ("lens", C.POINTER(C.c_uint64))]


class _Stats(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in ("lookups", "hits", "builds", "uncached_builds", "class_scans",
                                           "entries_walked", "keys", "cache_rows", "rows_in_use",
                                           "arena_bytes")]


class _StateInfo(C.Structure):
    _fields_ = [(k, C.c_uint32) for k in ("kind", "byte", "next_a", "next_b", "eos_next", "max",
                                           "tmpl", "n_keys", "key")]


class _Profile(C.Structure):
    _fields_ = [("fill_calls", C.c_uint64), ("advance_calls", C.c_uint64), ("lookup_ms", C.c_double),
                ("scan_ms", C.c_double), ("build_ms", C.c_double), ("gather_ms", C.c_double),
                ("advance_ms", C.c_double), ("apply_calls", C.c_uint64), ("apply_ms", C.c_double)]


EXPORTS = [
    "wg_vocab_create", "wg_vocab_destroy", "wg_lower", "wg_table_num_states",
    "wg_table_start_state", "wg_table_state", "wg_table_symbol_class", "wg_table_destroy",
    "wg_compile", "wg_destroy", "wg_num_states", "wg_mask_words", "wg_fill_masks",
    "wg_apply_mask", "wg_advance", "wg_cache_clear", "wg_cache_stats", "wg_error_count",
    "wg_last_error", "wg_select_tokens", "wg_profile_enable", "wg_profile_read", "wg_masked_argmax",
    "wg_add_instances", "wg_num_instances", "wg_cache_resize", "wg_table_add_instances",
    "wg_table_num_instances", "wg_advance_fill_masks", "wg_regex_to_template",
    "wg_decode_step", "wg_masked_topk", "wg_masked_topk_workspace", "wg_reserve_batch", "wg_max_batch", "wg_set_scan_batch",
    "wg_masked_topk_static", "wg_masked_topk_static_capacity", "wg_profile_apply_mask", "wg_forced_bytes",
]


def library_path():
    return _build.LIB


def load_library():
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            path + " is missing: build it first (python -m paper_2507_16768_amd.build)")
    L = C.CDLL(path)
    vp, u32, i32, u64, i64 = C.c_void_p, C.c_uint32, C.c_int32, C.c_uint64, C.c_int64
    L.wg_last_error.restype = C.c_char_p
    L.wg_vocab_create.argtypes = [vp, vp, u32, i32, C.POINTER(vp)]
    L.wg_vocab_destroy.argtypes = [vp]
    L.wg_vocab_destroy.restype = None
    L.wg_lower.argtypes = [C.POINTER(C.c_char_p), C.POINTER(_Args), u32, u32, u32, C.POINTER(vp)]
    L.wg_table_add_instances.argtypes = [vp, C.POINTER(C.c_char_p), C.POINTER(_Args), u32]
    L.wg_table_num_instances.argtypes = [vp]
    L.wg_table_num_instances.restype = u32
    L.wg_regex_to_template.argtypes = [C.c_char_p, C.c_char_p, u64, C.POINTER(u64)]
    L.wg_table_num_states.argtypes = [vp]
    L.wg_table_num_states.restype = u32
    L.wg_table_start_state.argtypes = [vp, u32]
    L.wg_table_start_state.restype = u32
    L.wg_table_state.argtypes = [vp, u32, C.POINTER(_StateInfo)]
    L.wg_table_symbol_class.argtypes = [vp, u32, u32]
    L.wg_table_destroy.argtypes = [vp]
    L.wg_table_destroy.restype = None
    L.wg_compile.argtypes = [C.POINTER(C.c_char_p), C.POINTER(_Args), u32, vp, u32, C.POINTER(vp), vp]
    L.wg_destroy.argtypes = [vp]
    L.wg_destroy.restype = None
    L.wg_add_instances.argtypes = [vp, C.POINTER(C.c_char_p), C.POINTER(_Args), u32, vp, vp]
    L.wg_num_instances.argtypes = [vp]
    L.wg_num_instances.restype = u32
    L.wg_cache_resize.argtypes = [vp, u32]
    L.wg_reserve_batch.argtypes = [vp, u32]
    L.wg_set_scan_batch.argtypes = [vp, u32]
    L.wg_max_batch.argtypes = [vp]
    L.wg_max_batch.restype = u32
    L.wg_num_states.argtypes = [vp]
    L.wg_num_states.restype = u32
    L.wg_mask_words.argtypes = [vp]
    L.wg_mask_words.restype = u32
    L.wg_fill_masks.argtypes = [vp, vp, u32, vp, vp]
    L.wg_apply_mask.argtypes = [vp, C.c_int, u32, u32, i64, vp, vp]
    L.wg_advance.argtypes = [vp, vp, vp, u32, vp]
    L.wg_advance_fill_masks.argtypes = [vp, vp, vp, u32, vp, vp]
    L.wg_decode_step.argtypes = [vp, vp, vp, u32, vp, vp, C.c_int, i64, vp]
    L.wg_masked_argmax.argtypes = [vp, C.c_int, u32, u32, i64, vp, vp, vp]
    L.wg_masked_topk_workspace.argtypes = [u32, u32, u32]
    L.wg_masked_topk_workspace.restype = u64
    L.wg_masked_topk.argtypes = [vp, C.c_int, u32, u32, i64, vp, u32, vp, vp, vp, u64, vp]
    L.wg_masked_topk_static_capacity.argtypes = []
    L.wg_masked_topk_static_capacity.restype = u64
    L.wg_masked_topk_static.argtypes = [vp, C.c_int, u32, u32, i64, vp, u32, vp, vp, vp]
    L.wg_forced_bytes.argtypes = [vp, vp, u32, u32, vp, vp, vp, vp]
    L.wg_cache_clear.argtypes = [vp, vp]
    L.wg_cache_stats.argtypes = [vp, C.POINTER(_Stats)]
    L.wg_error_count.argtypes = [vp, C.POINTER(u64)]
    L.wg_select_tokens.argtypes = [vp, u32, u32, vp, vp, vp]
    L.wg_profile_enable.argtypes = [vp, C.c_int]
    L.wg_profile_read.argtypes = [vp, C.POINTER(_Profile)]
    L.wg_profile_apply_mask.argtypes = [vp, vp, C.c_int, u32, u32, i64, vp, vp]
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise WgError(rc, load_library().wg_last_error().decode(errors="replace"))


def _marshal_templates(texts, args):
    n = len(texts)
    enc = [t.encode("utf-8") if isinstance(t, str) else bytes(t) for t in texts]
    c_texts = (C.c_char_p * max(n, 1))(*enc)
    keep = [enc, c_texts]
    c_args = None
    if args is not None:
        if len(args) != n:
            raise ValueError("one argument set per template is required")
        c_args = (_Args * max(n, 1))()
        for i, a in enumerate(args):
            names = [k.encode() for k in a]
            vals = [bytes(v) for v in a.values()]         # the C side reads the bytes objects' own storage
            m = len(names)
            c_names = (C.c_char_p * max(m, 1))(*names)
            c_data = (C.POINTER(C.c_uint8) * max(m, 1))(
                *[C.cast(C.c_char_p(v), C.POINTER(C.c_uint8)) for v in vals])
            c_lens = (C.c_uint64 * max(m, 1))(*[len(v) for v in vals])
            c_args[i] = _Args(m, c_names, c_data, c_lens)
            keep += [names, vals, c_names, c_data, c_lens]
        keep.append(c_args)
    return c_texts, c_args, n, keep


def marshal_templates(texts, args):
    """The C arrays of a list of templates and their argument sets, for add_instances(marshalled=...)."""
    return _marshal_templates(texts, args)


def _stream_ptr(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def _dev(t, dtype=None, name="tensor"):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(name + " must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s" % (name, dtype))
    return C.c_void_p(t.data_ptr())


def regex_to_template(regex):
    """wg_regex_to_template: template text (str) for a regular expression (str or bytes)."""
    L = load_library()
    rx = regex.encode("utf-8") if isinstance(regex, str) else bytes(regex)
    need = C.c_uint64(0)
    buf = C.create_string_buffer(4096)
    rc = L.wg_regex_to_template(rx, buf, len(buf), C.byref(need))
    if rc != 0 and need.value > len(buf):
        buf = C.create_string_buffer(need.value)
        rc = L.wg_regex_to_template(rx, buf, len(buf), C.byref(need))
    _check(rc)
    return buf.value.decode("latin-1")


class Table:
    """wg_lower: host-only lowering, for inspecting the state table without a GPU."""

    def __init__(self, texts, args=None, flags=EOS_STOP, lmax=0):
        L = load_library()
        c_texts, c_args, n, _keep = _marshal_templates(texts, args)
        self._t = C.c_void_p()
        _check(L.wg_lower(c_texts, c_args, n, flags, lmax, C.byref(self._t)))
        self.n_templates = n
        self.num_states = L.wg_table_num_states(self._t)

    def add_instances(self, texts, args=None):
        L = load_library()
        c_texts, c_args, n, _keep = _marshal_templates(texts, args)
        _check(L.wg_table_add_instances(self._t, c_texts, c_args, n))
        self.n_templates = L.wg_table_num_instances(self._t)
        self.num_states = L.wg_table_num_states(self._t)

    def start_state(self, i=0):
        return load_library().wg_table_start_state(self._t, i)

    def state(self, sid):
        info = _StateInfo()
        _check(load_library().wg_table_state(self._t, sid, C.byref(info)))
        return {k: getattr(info, k) for k, _ in _StateInfo._fields_}

    def symbol_class(self, sid, symbol):
        r = load_library().wg_table_symbol_class(self._t, sid, symbol)
        if r < 0:
            _check(r)
        return r

    def __del__(self):
        if getattr(self, "_t", None) and load_library is not None:   # (None: the interpreter is shutting down)
            load_library().wg_table_destroy(self._t)
            self._t = None


class Vocab:
    """wg_vocab_create: uploads CSR token bytes to HBM."""

    def __init__(self, token_bytes, offsets, eos_id):
        L = load_library()
        if isinstance(token_bytes, (bytes, bytearray)):
            token_bytes = np.frombuffer(bytes(token_bytes), dtype=np.uint8)
        b = np.ascontiguousarray(token_bytes, dtype=np.uint8)
        o = np.ascontiguousarray(offsets, dtype=np.uint64)
        self.V = len(o) - 1
        self.W = (self.V + 31) // 32
        self.eos_id = int(eos_id)
        self._v = C.c_void_p()
        _check(L.wg_vocab_create(b.ctypes.data, o.ctypes.data, self.V, self.eos_id, C.byref(self._v)))

    def __del__(self):
        if getattr(self, "_v", None) and load_library is not None:   # (None: the interpreter is shutting down)
            load_library().wg_vocab_destroy(self._v)
            self._v = None


class Handle:
    """wg_compile and the per-step calls on one set of template instances."""

    def __init__(self, texts, args, vocab, flags=EOS_RESTART):
        L = load_library()
        c_texts, c_args, n, _keep = _marshal_templates(texts, args)
        self.vocab = vocab                       # keeps the vocabulary alive
        starts = np.zeros((max(n, 1), 2), dtype=np.uint32)
        self._h = C.c_void_p()
        _check(L.wg_compile(c_texts, c_args, n, vocab._v, flags, C.byref(self._h), starts.ctypes.data))
        self.start_states = starts[:n]
        self.num_states = L.wg_num_states(self._h)
        self.W = L.wg_mask_words(self._h)

    def fill_masks(self, states, bitmask, stream=None):
        import torch
        B = states.shape[0]
        if tuple(states.shape) != (B, 2) or tuple(bitmask.shape) != (B, self.W):
            raise ValueError("states must be [B, 2] and bitmask [B, W]")
        _check(load_library().wg_fill_masks(self._h, _dev(states, torch.int32, "states"), B,
                                            _dev(bitmask, torch.int32, "bitmask"), _stream_ptr(stream)))

    def advance(self, states, tokens, stream=None):
        import torch
        B = states.shape[0]
        if tuple(states.shape) != (B, 2) or tuple(tokens.shape) != (B,):
            raise ValueError("states must be [B, 2] and tokens [B]")
        _check(load_library().wg_advance(self._h, _dev(states, torch.int32, "states"),
                                         _dev(tokens, torch.int32, "tokens"), B, _stream_ptr(stream)))

    def advance_fill_masks(self, states, tokens, bitmask, stream=None):
        import torch
        B = states.shape[0]
        if tuple(states.shape) != (B, 2) or tuple(tokens.shape) != (B,) or tuple(bitmask.shape) != (B, self.W):
            raise ValueError("states must be [B, 2], tokens [B] and bitmask [B, W]")
        _check(load_library().wg_advance_fill_masks(
            self._h, _dev(states, torch.int32, "states"), _dev(tokens, torch.int32, "tokens"), B,
            _dev(bitmask, torch.int32, "bitmask"), _stream_ptr(stream)))

    def decode_step(self, states, tokens, bitmask, logits, stream=None):
        """wg_decode_step; tokens may be None (first step)."""
        import torch
        B = states.shape[0]
        if tuple(states.shape) != (B, 2) or tuple(bitmask.shape) != (B, self.W):
            raise ValueError("states must be [B, 2] and bitmask [B, W]")
        if tokens is not None and tuple(tokens.shape) != (B,):
            raise ValueError("tokens must be [B]")
        if logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1 or logits.shape[0] != B:
            raise ValueError("logits must be a [B, V] device tensor with unit inner stride")
        if logits.shape[1] != self.vocab.V:
            raise ValueError("logits must have the vocabulary's width")
        dt = {torch.float32: F32, torch.bfloat16: BF16}.get(logits.dtype)
        if dt is None:
            raise ValueError("logits must be float32 or bfloat16")
        _check(load_library().wg_decode_step(
            self._h, _dev(states, torch.int32, "states"),
            None if tokens is None else _dev(tokens, torch.int32, "tokens"), B,
            _dev(bitmask, torch.int32, "bitmask"), C.c_void_p(logits.data_ptr()), dt, logits.stride(0),
            _stream_ptr(stream)))

    def forced_bytes(self, states, out_bytes, out_lens, end_states=None, stream=None):
        """wg_forced_bytes: out_bytes uint8 [B, cap], out_lens int32 [B], end_states int32 [B, 2] or None."""
        import torch
        B = states.shape[0]
        if tuple(states.shape) != (B, 2) or out_bytes.dim() != 2 or out_bytes.shape[0] != B or tuple(out_lens.shape) != (B,):
            raise ValueError("states must be [B, 2], out_bytes [B, cap] and out_lens [B]")
        if end_states is not None and tuple(end_states.shape) != (B, 2):
            raise ValueError("end_states must be [B, 2]")
        _check(load_library().wg_forced_bytes(
            self._h, _dev(states, torch.int32, "states"), B, out_bytes.shape[1],
            _dev(out_bytes, torch.uint8, "out_bytes"), _dev(out_lens, torch.int32, "out_lens"),
            None if end_states is None else _dev(end_states, torch.int32, "end_states"), _stream_ptr(stream)))

    def add_instances(self, texts, args, stream=None, marshalled=None):
        """wg_add_instances: returns the start states [n, 2] of the new instances.  `marshalled`
        takes what marshal_templates(texts, args) made beforehand instead of texts and args."""
        L = load_library()
        c_texts, c_args, n, _keep = marshalled if marshalled is not None else _marshal_templates(texts, args)
        starts = np.zeros((max(n, 1), 2), dtype=np.uint32)
        _check(L.wg_add_instances(self._h, c_texts, c_args, n, starts.ctypes.data, _stream_ptr(stream)))
        self.start_states = np.concatenate([self.start_states, starts[:n]])
        self.num_states = L.wg_num_states(self._h)
        return starts[:n]

    def num_instances(self):
        return load_library().wg_num_instances(self._h)

    def reserve_batch(self, max_batch):
        _check(load_library().wg_reserve_batch(self._h, int(max_batch)))

    def max_batch(self):
        return load_library().wg_max_batch(self._h)

    def set_scan_batch(self, tables):
        _check(load_library().wg_set_scan_batch(self._h, int(tables)))

    def cache_resize(self, rows):
        _check(load_library().wg_cache_resize(self._h, int(rows)))

    def cache_clear(self, stream=None):
        _check(load_library().wg_cache_clear(self._h, _stream_ptr(stream)))

    def cache_stats(self):
        s = _Stats()
        _check(load_library().wg_cache_stats(self._h, C.byref(s)))
        return {k: getattr(s, k) for k, _ in _Stats._fields_}

    def profile_enable(self, on=True):
        _check(load_library().wg_profile_enable(self._h, 1 if on else 0))

    def profile_read(self):
        p = _Profile()
        _check(load_library().wg_profile_read(self._h, C.byref(p)))
        return {k: getattr(p, k) for k, _ in _Profile._fields_}

    def profile_apply_mask(self, logits, bitmask, stream=None):
        """wg_profile_apply_mask: wg_apply_mask, timed into this handle's record while timing is enabled."""
        import torch
        dt = {torch.float32: F32, torch.bfloat16: BF16}.get(logits.dtype)
        if dt is None or logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1:
            raise ValueError("logits must be a [B, V] float32 or bfloat16 device tensor with unit inner stride")
        B, V = logits.shape
        if tuple(bitmask.shape) != (B, (V + 31) // 32):
            raise ValueError("bitmask must be [B, ceil(V/32)]")
        _check(load_library().wg_profile_apply_mask(self._h, C.c_void_p(logits.data_ptr()), dt, B, V, logits.stride(0),
                                                    _dev(bitmask, torch.int32, "bitmask"), _stream_ptr(stream)))

    def error_count(self):
        n = C.c_uint64()
        _check(load_library().wg_error_count(self._h, C.byref(n)))
        return n.value

    def __del__(self):
        if getattr(self, "_h", None) and load_library is not None:   # (None: the interpreter is shutting down)
            load_library().wg_destroy(self._h)
            self._h = None


def apply_mask(logits, bitmask, stream=None):
    """wg_apply_mask on a [B, V] float32 or bfloat16 device tensor (rows may be strided)."""
    import torch
    if logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits must be a 2-d device tensor with unit inner stride")
    if logits.dtype == torch.float32:
        dt = F32
    elif logits.dtype == torch.bfloat16:
        dt = BF16
    else:
        raise ValueError("logits must be float32 or bfloat16")
    B, V = logits.shape
    if tuple(bitmask.shape) != (B, (V + 31) // 32):
        raise ValueError("bitmask must be [B, ceil(V/32)]")
    _check(load_library().wg_apply_mask(C.c_void_p(logits.data_ptr()), dt, B, V, logits.stride(0),
                                        _dev(bitmask, torch.int32, "bitmask"), _stream_ptr(stream)))


def masked_argmax(logits, bitmask, tokens, stream=None):
    """wg_masked_argmax on a [B, V] float32 or bfloat16 device tensor; tokens is int32 [B]."""
    import torch
    if logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits must be a 2-d device tensor with unit inner stride")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(logits.dtype)
    if dt is None:
        raise ValueError("logits must be float32 or bfloat16")
    B, V = logits.shape
    if tuple(bitmask.shape) != (B, (V + 31) // 32) or tuple(tokens.shape) != (B,):
        raise ValueError("bitmask must be [B, ceil(V/32)] and tokens [B]")
    _check(load_library().wg_masked_argmax(C.c_void_p(logits.data_ptr()), dt, B, V, logits.stride(0),
                                           _dev(bitmask, torch.int32, "bitmask"),
                                           _dev(tokens, torch.int32, "tokens"), _stream_ptr(stream)))


def masked_topk_workspace(B, V, k):
    """wg_masked_topk_workspace: bytes of device workspace a wg_masked_topk call of this shape needs."""
    return int(load_library().wg_masked_topk_workspace(B, V, k))


def masked_topk(logits, bitmask, ids, values, workspace, stream=None):
    """wg_masked_topk on a [B, V] float32 or bfloat16 device tensor: ids is int32 [B, k], values
    [B, k] of the logits' dtype, workspace a device tensor of at least masked_topk_workspace bytes."""
    import torch
    if logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits must be a 2-d device tensor with unit inner stride")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(logits.dtype)
    if dt is None:
        raise ValueError("logits must be float32 or bfloat16")
    B, V = logits.shape
    if ids.dim() != 2 or ids.shape[0] != B or tuple(values.shape) != tuple(ids.shape):
        raise ValueError("ids and values must be [B, k]")
    if tuple(bitmask.shape) != (B, (V + 31) // 32):
        raise ValueError("bitmask must be [B, ceil(V/32)]")
    _check(load_library().wg_masked_topk(C.c_void_p(logits.data_ptr()), dt, B, V, logits.stride(0),
                                         _dev(bitmask, torch.int32, "bitmask"), ids.shape[1],
                                         _dev(ids, torch.int32, "ids"), _dev(values, logits.dtype, "values"),
                                         _dev(workspace, None, "workspace"),
                                         workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


def masked_topk_static_capacity():
    """wg_masked_topk_static_capacity: bytes of lists the library holds per GPU."""
    return int(load_library().wg_masked_topk_static_capacity())


def masked_topk_static(logits, bitmask, ids, values, stream=None):
    """wg_masked_topk_static: wg_masked_topk with the library's own workspace (nothing allocated)."""
    import torch
    if logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits must be a 2-d device tensor with unit inner stride")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(logits.dtype)
    if dt is None:
        raise ValueError("logits must be float32 or bfloat16")
    B, V = logits.shape
    if ids.dim() != 2 or ids.shape[0] != B or tuple(values.shape) != tuple(ids.shape):
        raise ValueError("ids and values must be [B, k]")
    if tuple(bitmask.shape) != (B, (V + 31) // 32):
        raise ValueError("bitmask must be [B, ceil(V/32)]")
    _check(load_library().wg_masked_topk_static(C.c_void_p(logits.data_ptr()), dt, B, V, logits.stride(0),
                                                _dev(bitmask, torch.int32, "bitmask"), ids.shape[1],
                                                _dev(ids, torch.int32, "ids"), _dev(values, logits.dtype, "values"),
                                                _stream_ptr(stream)))


def select_tokens(bitmask, V, draws, tokens, stream=None):
    """wg_select_tokens: harness sampler stand-in."""
    import torch
    B = bitmask.shape[0]
    _check(load_library().wg_select_tokens(_dev(bitmask, torch.int32, "bitmask"), B, V,
                                           _dev(draws, torch.int64, "draws"),
                                           _dev(tokens, torch.int32, "tokens"), _stream_ptr(stream)))
