"""ctypes binding of include/zapformat.h.

Only marshals arguments: every step of the hot path runs inside the library.  The
library must have been built (paper_2506_01151_amd/build.py); a missing library is
an error, there is no substitute path.
"""
import ctypes
import os
import numpy as np

ZF_OK, ZF_ERR_INVALID_ARG, ZF_ERR_GRAMMAR, ZF_ERR_REJECTED = 0, -1, -2, -3
ZF_ERR_RANGE, ZF_ERR_DEVICE, ZF_ERR_OOM, ZF_ERR_OVERFLOW = -4, -5, -6, -7

_HERE = os.path.dirname(os.path.abspath(__file__))
# ZAPFORMAT_LIBRARY names another build of the same library (the sanitizer build of paper_2506_01151_amd/build.py --sanitize)
LIB_PATH = os.environ.get("ZAPFORMAT_LIBRARY") or os.path.join(_HERE, "libzapformat.so")
_lib = None

c_i32, c_i64, c_vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p


class GrammarDesc(ctypes.Structure):
    _fields_ = [("n_nonterminals", c_i32), ("start", c_i32), ("n_rules", c_i32),
                ("rule_lhs", c_vp), ("rhs_off", c_vp), ("rhs_sym", c_vp),
                ("n_terminals", c_i32), ("term_kind", c_vp), ("term_off", c_vp), ("term_data", c_vp)]


class VocabDesc(ctypes.Structure):
    _fields_ = [("V", c_i32), ("off", c_vp), ("bytes", c_vp)]


class Options(ctypes.Structure):
    _fields_ = [("pruning", c_i32), ("lane_item_cap", c_i32), ("device", c_i32), ("chunk_strings", c_i32), ("fallback_item_cap", c_i32), ("state_cache_entries", c_i32), ("disable_token_mask_cache", c_i32), ("walk_mode", c_i32), ("precompute_states", c_i32)]


class Stats(ctypes.Structure):
    _fields_ = [("n_sets", c_i64), ("n_items", c_i64), ("items_created", c_i64), ("bytes_fed", c_i64),
                ("accepting", c_i32)]


class EngineInfo(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("V", "W", "n_nonterminals", "n_rules", "n_positions", "n_dfa_states",
                                     "n_byte_classes", "n_trie_nodes", "n_strings", "lane_item_cap", "device", "table_lds_mode")]


class MaskReport(ctypes.Structure):
    _fields_ = [("overflow_chunks", c_i64), ("walk_chunks", c_i64), ("chart_bytes", c_i64), ("cache_hits", c_i32), ("cache_misses", c_i32), ("main_ms", ctypes.c_float),
                ("fallback_ms", ctypes.c_float), ("permute_ms", ctypes.c_float), ("parser_steps", c_i32), ("cache_rows", c_i32)]


EXPORTS = ["zf_strerror", "zf_last_error", "zf_compile", "zf_engine_destroy", "zf_engine_get_info",
           "zf_state_new", "zf_state_clone", "zf_state_reset", "zf_state_destroy", "zf_advance",
           "zf_advance_bytes", "zf_advance_batch", "zf_is_accepting", "zf_state_stats", "zf_state_chart", "zf_position_info",
           "zf_compute_mask", "zf_compute_mask_noalloc", "zf_compute_mask_async", "zf_compute_mask_apply_async", "zf_mask_wait", "zf_last_mask_report", "zf_engine_clear_state_cache", "zf_engine_set_profiling", "zf_apply_mask"]
# test-only diagnostics (include/zapformat_debug.h)
DEBUG_EXPORTS = ["zf_debug_host_mask", "zf_debug_host_mask_stats", "zf_debug_host_mask_cached", "zf_debug_host_mask_automaton",
                 "zf_debug_twin_new", "zf_debug_twin_destroy", "zf_debug_twin_advance", "zf_debug_twin_mask"]


class ZfError(RuntimeError):
    def __init__(self, code, detail):
        super().__init__(f"zapformat error {code}: {detail}")
        self.code = code


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2506_01151_amd/build.py`")
    L = ctypes.CDLL(LIB_PATH)
    L.zf_strerror.restype = ctypes.c_char_p
    L.zf_strerror.argtypes = [ctypes.c_int]
    L.zf_last_error.restype = ctypes.c_char_p
    L.zf_compile.argtypes = [c_vp, c_vp, c_vp, ctypes.POINTER(c_vp)]
    L.zf_engine_destroy.argtypes = [c_vp]
    L.zf_engine_destroy.restype = None
    L.zf_engine_get_info.argtypes = [c_vp, c_vp]
    L.zf_state_new.argtypes = [c_vp, ctypes.POINTER(c_vp)]
    L.zf_state_clone.argtypes = [c_vp, ctypes.POINTER(c_vp)]
    L.zf_state_reset.argtypes = [c_vp]
    L.zf_state_destroy.argtypes = [c_vp]
    L.zf_state_destroy.restype = None
    L.zf_advance.argtypes = [c_vp, c_i32]
    L.zf_advance_bytes.argtypes = [c_vp, c_vp, c_i64]
    L.zf_is_accepting.argtypes = [c_vp, ctypes.POINTER(c_i32)]
    L.zf_state_stats.argtypes = [c_vp, c_vp]
    L.zf_state_chart.argtypes = [c_vp, c_vp, c_vp]
    L.zf_position_info.argtypes = [c_vp, c_i32, ctypes.POINTER(c_i32), ctypes.POINTER(c_i32), ctypes.POINTER(c_i32)]
    L.zf_compute_mask.argtypes = [c_vp, c_vp, c_i32, c_vp, c_vp]
    L.zf_compute_mask_async.argtypes = [c_vp, c_vp, c_i32, c_vp, c_vp]
    L.zf_compute_mask_noalloc.argtypes = [c_vp, c_vp, c_i32, c_vp, c_vp]
    L.zf_compute_mask_apply_async.argtypes = [c_vp, c_vp, c_i32, c_vp, c_vp, c_vp, c_i32, c_i64, c_vp]
    L.zf_mask_wait.argtypes = [c_vp, c_vp]
    L.zf_last_mask_report.argtypes = [c_vp, c_vp]
    L.zf_advance_batch.argtypes = [c_vp, c_vp, c_i32, c_vp]
    L.zf_engine_set_profiling.argtypes = [c_vp, c_i32]
    L.zf_engine_clear_state_cache.argtypes = [c_vp]
    L.zf_apply_mask.argtypes = [c_vp, c_vp, c_vp, c_i32, c_i32, c_i64, c_vp, c_vp]
    L.zf_debug_host_mask.argtypes = [c_vp, c_vp, c_vp]
    L.zf_debug_host_mask_stats.argtypes = [c_vp, c_vp, c_vp, c_vp]
    L.zf_debug_host_mask_cached.argtypes = [c_vp, c_vp, c_vp, c_vp]
    L.zf_debug_host_mask_automaton.argtypes = [c_vp, c_vp, c_vp, c_vp]
    L.zf_debug_twin_new.argtypes = [c_vp, ctypes.POINTER(c_vp)]
    L.zf_debug_twin_destroy.argtypes = [c_vp]
    L.zf_debug_twin_destroy.restype = None
    L.zf_debug_twin_advance.argtypes = [c_vp, ctypes.POINTER(ctypes.c_uint32), c_vp, c_i64, ctypes.POINTER(c_i32)]
    L.zf_debug_twin_mask.argtypes = [c_vp, ctypes.c_uint32, c_vp, c_vp]
    _lib = L
    return L


def _check(rc):
    if rc != ZF_OK:
        raise ZfError(rc, _lib.zf_last_error().decode("utf-8", "replace"))


class State:
    def __init__(self, engine, handle):
        self.engine, self.h = engine, handle

    def __del__(self):
        if self.h and _lib is not None:
            _lib.zf_state_destroy(self.h)
            self.h = None

    def clone(self):
        h = c_vp()
        _check(_lib.zf_state_clone(self.h, ctypes.byref(h)))
        return State(self.engine, h)

    def reset(self):
        _check(_lib.zf_state_reset(self.h))

    def advance(self, token_id: int):
        _check(_lib.zf_advance(self.h, token_id))

    def try_advance(self, token_id: int) -> int:
        return _lib.zf_advance(self.h, token_id)

    def advance_bytes(self, data: bytes):
        buf = (ctypes.c_uint8 * max(1, len(data))).from_buffer_copy(data or b"\0")
        _check(_lib.zf_advance_bytes(self.h, buf, len(data)))

    def try_advance_bytes(self, data: bytes) -> int:
        buf = (ctypes.c_uint8 * max(1, len(data))).from_buffer_copy(data or b"\0")
        return _lib.zf_advance_bytes(self.h, buf, len(data))

    def accepting(self) -> bool:
        out = c_i32()
        _check(_lib.zf_is_accepting(self.h, ctypes.byref(out)))
        return bool(out.value)

    def stats(self) -> Stats:
        s = Stats()
        _check(_lib.zf_state_stats(self.h, ctypes.byref(s)))
        return s

    def chart(self):
        """[(set index, dotted position, origin, dfa state)] plus the number of sets."""
        st = self.stats()
        items = np.zeros((max(1, st.n_items), 3), dtype=np.int32)
        off = np.zeros(st.n_sets + 1, dtype=np.int64)
        _check(_lib.zf_state_chart(self.h, items.ctypes.data, off.ctypes.data))
        out = []
        for k in range(st.n_sets):
            for i in range(off[k], off[k + 1]):
                out.append((k, int(items[i, 0]), int(items[i, 1]), int(items[i, 2])))
        return out, int(st.n_sets)

    def debug_host_mask_stats(self):
        out = np.zeros(self.engine.W, dtype=np.uint32)
        st = np.zeros(8, dtype=np.int64)
        _check(_lib.zf_debug_host_mask_stats(self.engine.h, self.h, out.ctypes.data, st.ctypes.data))
        return out, dict(steps=int(st[0]), alive=int(st[1]), max_path=int(st[2]), max_set=int(st[3]), chunks_over=int(st[4]))

    def debug_host_mask_cached(self):
        out = np.zeros(self.engine.W, dtype=np.uint32)
        st = np.zeros(8, dtype=np.int64)
        _check(_lib.zf_debug_host_mask_cached(self.engine.h, self.h, out.ctypes.data, st.ctypes.data))
        return out, dict(steps=int(st[0]), undecided=int(st[1]), cache_rows=int(st[2]), replay_steps=int(st[3]), chunks=int(st[4]))

    def debug_host_mask_automaton(self):
        out = np.zeros(self.engine.W, dtype=np.uint32)
        st = np.zeros(8, dtype=np.int64)
        _check(_lib.zf_debug_host_mask_automaton(self.engine.h, self.h, out.ctypes.data, st.ctypes.data))
        return out, dict(states=int(st[0]), steps=int(st[1]), lookups=int(st[2]), undecided=int(st[3]), max_set=int(st[4]))

    def debug_host_mask(self) -> np.ndarray:
        out = np.zeros(self.engine.W, dtype=np.uint32)
        _check(_lib.zf_debug_host_mask(self.engine.h, self.h, out.ctypes.data))
        return out


class Twin:
    """Test-only: host twin of the persistent automaton (include/zapformat_debug.h)."""

    def __init__(self, engine):
        self.engine = engine
        h = c_vp()
        _check(_lib.zf_debug_twin_new(engine.h, ctypes.byref(h)))
        self.h = h

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.zf_debug_twin_destroy(self.h)
            self.h = None

    def advance(self, state: int, data: bytes):
        """(return code, next state, accepting)."""
        buf = (ctypes.c_uint8 * max(1, len(data))).from_buffer_copy(data or b"\0")
        st, acc = ctypes.c_uint32(state), c_i32()
        rc = _lib.zf_debug_twin_advance(self.h, ctypes.byref(st), buf, len(data), ctypes.byref(acc))
        return rc, st.value, bool(acc.value)

    def mask(self, state: int):
        out = np.zeros(self.engine.W, dtype=np.uint32)
        st = np.zeros(8, dtype=np.int64)
        _check(_lib.zf_debug_twin_mask(self.h, state, out.ctypes.data, st.ctypes.data))
        return out, dict(states=int(st[0]), steps=int(st[1]), lookups=int(st[2]), undecided=int(st[3]), items=int(st[4]))


class StateBatch:
    """The rows of one batch with their handle array marshalled once: pass it wherever a list of
    states is accepted; advance() moves every row by one token in a single library call."""

    def __init__(self, states):
        self.states = list(states)
        self.arr = (c_vp * max(1, len(self.states)))(*[s.h for s in self.states])
        self._ids = (c_i32 * max(1, len(self.states)))()

    def __len__(self):
        return len(self.states)

    def __getitem__(self, i):
        return self.states[i]

    def __iter__(self):
        return iter(self.states)

    def advance(self, token_ids):
        """token_ids[b] < 0 resets row b."""
        self._ids[:len(self.states)] = token_ids
        _check(_lib.zf_advance_batch(self.arr, self._ids, len(self.states), None))


def _handles(states):
    return states.arr if isinstance(states, StateBatch) else (c_vp * len(states))(*[s.h for s in states])


class Engine:
    """compile(grammar rules, vocab byte strings)."""

    def __init__(self, grammar, vocab_tokens, *, pruning=True, lane_item_cap=0, device=0, chunk_strings=0, fallback_item_cap=0, token_mask_cache=True, state_cache_entries=0, walk_mode=2, precompute_states=0):
        load_library()
        csr = grammar.csr()
        self._keep = csr
        gd = GrammarDesc(csr["n_nonterminals"], csr["start"], len(csr["rule_lhs"]),
                         csr["rule_lhs"].ctypes.data, csr["rhs_off"].ctypes.data, csr["rhs_sym"].ctypes.data,
                         len(csr["term_kind"]), csr["term_kind"].ctypes.data, csr["term_off"].ctypes.data,
                         csr["term_data"].ctypes.data)
        off = np.zeros(len(vocab_tokens) + 1, dtype=np.int64)
        np.cumsum([len(t) for t in vocab_tokens], out=off[1:])
        data = np.frombuffer(b"".join(vocab_tokens) or b"\0", dtype=np.uint8).copy()
        vd = VocabDesc(len(vocab_tokens), off.ctypes.data, data.ctypes.data)
        opt = Options(int(bool(pruning)), lane_item_cap, device, chunk_strings, fallback_item_cap, state_cache_entries, int(not token_mask_cache), walk_mode, precompute_states)
        h = c_vp()
        self.h = None
        _check(_lib.zf_compile(ctypes.byref(gd), ctypes.byref(vd), ctypes.byref(opt), ctypes.byref(h)))
        self.h = h
        self.info = EngineInfo()
        _check(_lib.zf_engine_get_info(self.h, ctypes.byref(self.info)))
        self.V, self.W = self.info.V, self.info.W

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.zf_engine_destroy(self.h)
            self.h = None

    def new_state(self) -> State:
        h = c_vp()
        _check(_lib.zf_state_new(self.h, ctypes.byref(h)))
        return State(self, h)

    def position_info(self, p):
        a, b, c = c_i32(), c_i32(), c_i32()
        _check(_lib.zf_position_info(self.h, p, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        return a.value, b.value, c.value

    def compute_mask(self, states, d_mask_ptr: int, stream: int = 0):
        _check(_lib.zf_compute_mask(self.h, _handles(states), len(states), d_mask_ptr, stream))

    def compute_mask_noalloc(self, states, d_mask_ptr: int, stream: int = 0):
        _check(_lib.zf_compute_mask_noalloc(self.h, _handles(states), len(states), d_mask_ptr, stream))

    def compute_mask_async(self, states, d_mask_ptr: int, stream: int = 0):
        _check(_lib.zf_compute_mask_async(self.h, _handles(states), len(states), d_mask_ptr, stream))

    def compute_mask_apply_async(self, states, d_mask_ptr: int, d_logits_ptr: int, d_out_ptr: int, dtype: int, row_stride: int, stream: int = 0):
        _check(_lib.zf_compute_mask_apply_async(self.h, _handles(states), len(states), d_mask_ptr, d_logits_ptr, d_out_ptr, dtype, row_stride, stream))

    def mask_wait(self, stream: int = 0):
        _check(_lib.zf_mask_wait(self.h, stream))

    def clear_state_cache(self):
        _check(_lib.zf_engine_clear_state_cache(self.h))

    def set_profiling(self, on: bool):
        _check(_lib.zf_engine_set_profiling(self.h, int(on)))

    def mask_report(self) -> MaskReport:
        r = MaskReport()
        _check(_lib.zf_last_mask_report(self.h, ctypes.byref(r)))
        return r

    def apply_mask(self, d_logits_ptr: int, d_out_ptr: int, dtype: int, batch: int, row_stride: int,
                   d_mask_ptr: int, stream: int = 0):
        _check(_lib.zf_apply_mask(self.h, d_logits_ptr, d_out_ptr, dtype, batch, row_stride, d_mask_ptr, stream))


# the four calls by their names in the problem statement --------------------------------
def compile(grammar, vocab_tokens, **kw) -> Engine:
    return Engine(grammar, vocab_tokens, **kw)


def advance(state: State, token_id: int):
    state.advance(token_id)


def _current_stream(engine: Engine) -> int:
    """Handle of torch's current stream on the engine's device (what the library enqueues on)."""
    import torch
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)   # the same handle without building a Stream object
    if raw is not None:
        return raw(engine.info.device)
    return torch.cuda.current_stream(engine.info.device).cuda_stream


def compute_mask(engine: Engine, states, mask_tensor):
    """mask_tensor: torch int32 tensor [batch, W] on the engine's device (fully overwritten)."""
    import torch
    assert mask_tensor.is_cuda and mask_tensor.is_contiguous() and mask_tensor.dtype == torch.int32
    assert tuple(mask_tensor.shape) == (len(states), engine.W)
    engine.compute_mask(states, mask_tensor.data_ptr(), _current_stream(engine))
    return mask_tensor


def compute_mask_noalloc(engine: Engine, states, mask_tensor):
    """compute_mask through the entry point that allocates no device memory (static scratch array)."""
    import torch
    assert mask_tensor.is_cuda and mask_tensor.is_contiguous() and mask_tensor.dtype == torch.int32
    assert tuple(mask_tensor.shape) == (len(states), engine.W)
    engine.compute_mask_noalloc(states, mask_tensor.data_ptr(), _current_stream(engine))
    return mask_tensor


def compute_mask_async(engine: Engine, states, mask_tensor):
    """Enqueue only; pair with mask_wait(engine) before reading the mask on the host."""
    import torch
    assert mask_tensor.is_cuda and mask_tensor.is_contiguous() and mask_tensor.dtype == torch.int32
    assert tuple(mask_tensor.shape) == (len(states), engine.W)
    engine.compute_mask_async(states, mask_tensor.data_ptr(), _current_stream(engine))
    return mask_tensor


def compute_mask_apply_async(engine: Engine, states, mask_tensor, logits, out=None):
    """compute_mask and apply_mask of the same rows, enqueued together; pair with mask_wait(engine)."""
    import torch
    assert mask_tensor.is_cuda and mask_tensor.is_contiguous() and mask_tensor.dtype == torch.int32
    assert tuple(mask_tensor.shape) == (len(states), engine.W)
    assert logits.is_cuda and logits.dim() == 2 and logits.stride(1) == 1 and tuple(logits.shape) == (len(states), engine.V)
    dtype = {torch.float32: 0, torch.bfloat16: 1}[logits.dtype]
    if out is None:
        out = logits
    assert out.dtype == logits.dtype and out.shape == logits.shape and out.stride() == logits.stride()
    engine.compute_mask_apply_async(states, mask_tensor.data_ptr(), logits.data_ptr(), out.data_ptr(), dtype, logits.stride(0), _current_stream(engine))
    return out


def mask_wait(engine: Engine):
    engine.mask_wait(_current_stream(engine))


def apply_mask(engine: Engine, logits, mask_tensor, out=None):
    """logits: torch fp32 or bf16 tensor [batch, V] (last dim contiguous) on the device."""
    import torch
    assert logits.is_cuda and logits.dim() == 2 and logits.stride(1) == 1 and logits.shape[1] == engine.V
    dtype = {torch.float32: 0, torch.bfloat16: 1}[logits.dtype]
    if out is None:
        out = logits
    assert out.dtype == logits.dtype and out.shape == logits.shape and out.stride() == logits.stride()
    engine.apply_mask(logits.data_ptr(), out.data_ptr(), dtype, logits.shape[0], logits.stride(0),
                      mask_tensor.data_ptr(), _current_stream(engine))
    return out
