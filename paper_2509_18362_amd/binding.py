"""Thin ctypes binding of libmtp_draft.so: same names as the C ABI (include/mtp_draft.h), argument marshalling only.

Tensors are passed as torch CUDA tensors (or raw integer addresses); PyTorch supplies device memory and streams,
every step of the draft path runs inside the library's HIP kernels.  There is no fallback: if the library is not
built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

# PyTorch first: it ships its own copy of the HIP runtime and loads it by path.  Loaded afterwards, this library's
# dependency on the runtime resolves to that copy; loaded before it, the system's copy would come in as a second
# runtime in the same process, which then finds no device.
import torch  # noqa: F401  (isort: keep above the CDLL call)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmtp_draft.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python paper_2509_18362_amd/build.py) first; there is no CPU fallback")
_lib = C.CDLL(LIB_PATH)

MTP_OK = 0
STATUS = {0: "MTP_OK", -1: "MTP_ERR_NULL", -2: "MTP_ERR_ALIGN", -3: "MTP_ERR_CONFIG", -4: "MTP_ERR_BATCH",
          -5: "MTP_ERR_STEPS", -6: "MTP_ERR_SUBSET", -7: "MTP_ERR_WORKSPACE", -8: "MTP_ERR_HIP",
          -9: "MTP_ERR_KV_OVERFLOW", -10: "MTP_ERR_TOKEN_RANGE", -11: "MTP_ERR_MODE", -12: "MTP_ERR_TIMEOUT"}
EXPORTS = ["mtp_status_string", "mtp_workspace_bytes", "mtp_draft_init", "mtp_draft_steps", "mtp_draft_extend",
           "mtp_draft_continue", "mtp_draft_steps_lists", "mtp_subset_workspace_bytes", "mtp_subset_build",
           "mtp_subset_static_max_vocab", "mtp_subset_build_static",
           "mtp_train_workspace_bytes", "mtp_train_loss",
           "mtp_accept",
           "mtp_poll_error", "mtp_set_timing", "mtp_last_draft_ms", "mtp_set_launch_mode", "mtp_set_phase_trace",
           "mtp_phase_trace_bytes", "mtp_stream_probe",
           "mtp_draft_destroy"]
LAUNCH_PER_PHASE, LAUNCH_SINGLE, LAUNCH_AUTO, LAUNCH_ROWS = 0, 1, 2, 3
# mtp_set_timing modes
TIMING_OFF, TIMING_CALL = 0, 1
PHASES = ["proj", "qkv", "attn", "oproj", "gateup", "down", "lmhead"]


def timing_phase(name: str) -> int:
    return 2 + PHASES.index(name)


class mtp_config(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("max_batch", C.c_int32),
                ("kv_capacity", C.c_int32), ("max_draft_steps", C.c_int32)]


WEIGHT_FIELDS = ["embed", "lm_head", "g_hnorm", "g_enorm", "g_attn_norm", "g_mlp_norm", "g_final_norm", "w_proj",
                 "w_q", "w_k", "w_v", "b_q", "b_k", "b_v", "w_o", "w_gate", "w_up", "w_down"]


class mtp_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


_lib.mtp_status_string.restype = C.c_char_p
_lib.mtp_status_string.argtypes = [C.c_int32]
_lib.mtp_workspace_bytes.restype = C.c_size_t
_lib.mtp_workspace_bytes.argtypes = [C.POINTER(mtp_config)]
_lib.mtp_draft_init.restype = C.c_int32
_lib.mtp_draft_init.argtypes = [C.POINTER(C.c_void_p), C.POINTER(mtp_config), C.POINTER(mtp_weights), C.c_int32,
                                C.POINTER(C.c_void_p), C.POINTER(C.c_int32), C.c_void_p, C.c_size_t]
_lib.mtp_draft_steps.restype = C.c_int32
_lib.mtp_draft_steps.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 10
_lib.mtp_subset_workspace_bytes.restype = C.c_size_t
_lib.mtp_subset_workspace_bytes.argtypes = [C.c_int32]
_lib.mtp_subset_build.restype = C.c_int32
_lib.mtp_subset_build.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
_lib.mtp_subset_static_max_vocab.restype = C.c_int32
_lib.mtp_subset_static_max_vocab.argtypes = []
_lib.mtp_subset_build_static.restype = C.c_int32
_lib.mtp_subset_build_static.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
_lib.mtp_train_workspace_bytes.restype = C.c_size_t
_lib.mtp_train_workspace_bytes.argtypes = [C.c_void_p, C.c_int32]
_lib.mtp_train_loss.restype = C.c_int32
_lib.mtp_train_loss.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
_lib.mtp_draft_steps_lists.restype = C.c_int32
_lib.mtp_draft_steps_lists.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)] + [C.c_void_p] * 10
_lib.mtp_draft_continue.restype = C.c_int32
_lib.mtp_draft_continue.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 10
_lib.mtp_draft_extend.restype = C.c_int32
_lib.mtp_draft_extend.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 10
_lib.mtp_accept.restype = C.c_int32
_lib.mtp_accept.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32] + [C.c_void_p] * 5
_lib.mtp_poll_error.restype = C.c_int32
_lib.mtp_poll_error.argtypes = [C.c_void_p, C.c_void_p]
_lib.mtp_set_timing.restype = C.c_int32
_lib.mtp_set_timing.argtypes = [C.c_void_p, C.c_int32]
_lib.mtp_last_draft_ms.restype = C.c_float
_lib.mtp_last_draft_ms.argtypes = [C.c_void_p]
_lib.mtp_set_launch_mode.restype = C.c_int32
_lib.mtp_set_launch_mode.argtypes = [C.c_void_p, C.c_int32]
_lib.mtp_stream_probe.restype = C.c_int32
_lib.mtp_stream_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
_lib.mtp_phase_trace_bytes.restype = C.c_size_t
_lib.mtp_phase_trace_bytes.argtypes = [C.POINTER(mtp_config)]
_lib.mtp_set_phase_trace.restype = C.c_int32
_lib.mtp_set_phase_trace.argtypes = [C.c_void_p, C.c_void_p]
_lib.mtp_draft_destroy.restype = None
_lib.mtp_draft_destroy.argtypes = [C.c_void_p]


def _addr(t) -> Optional[int]:
    """Device address of a torch tensor, an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def make_config(shape, max_batch: int, kv_capacity: int, max_draft_steps: int) -> mtp_config:
    return mtp_config(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                      shape.vocab_size, shape.rms_eps, shape.rope_theta, max_batch, kv_capacity, max_draft_steps)


def mtp_status_string(status: int) -> str:
    return _lib.mtp_status_string(status).decode()


def mtp_workspace_bytes(cfg: mtp_config) -> int:
    return int(_lib.mtp_workspace_bytes(C.byref(cfg)))


def mtp_draft_init(cfg: mtp_config, weights: Dict[str, object], subsets: Sequence[object],
                   subset_sizes: Sequence[int], workspace, workspace_bytes: int):
    """Returns (status, handle).  weights: name -> device tensor/address (biases optional)."""
    w = mtp_weights(**{n: _addr(weights.get(n)) for n in WEIGHT_FIELDS})
    ns = len(subsets)
    ids = (C.c_void_p * max(ns, 1))(*[_addr(s) for s in subsets])
    sizes = (C.c_int32 * max(ns, 1))(*[int(s) for s in subset_sizes])
    handle = C.c_void_p(None)
    st = _lib.mtp_draft_init(C.byref(handle), C.byref(cfg), C.byref(w), ns, ids if ns else None,
                             sizes if ns else None, _addr(workspace), workspace_bytes)
    return int(st), (handle if st == MTP_OK else None)


def mtp_draft_steps_lists(handle, B: int, K: int, seq_subset, hidden_in, token_in, k_cache, v_cache, kv_len,
                          forced_tokens, draft_out, logits_out=None, hidden_out=None, stream=0) -> int:
    """seq_subset: a host sequence of B list indices."""
    arr = (C.c_int32 * B)(*[int(x) for x in seq_subset])
    return int(_lib.mtp_draft_steps_lists(handle, B, K, arr, _addr(hidden_in), _addr(token_in), _addr(k_cache),
                                          _addr(v_cache), _addr(kv_len), _addr(forced_tokens), _addr(draft_out),
                                          _addr(logits_out), _addr(hidden_out), stream))


def mtp_subset_workspace_bytes(vocab_size: int) -> int:
    return int(_lib.mtp_subset_workspace_bytes(vocab_size))


def mtp_subset_build(tokens, n_tokens: int, vocab_size: int, n: int, workspace, workspace_bytes: int, ids_out,
                     counts_out=None, invalid_out=None, stream=0) -> int:
    return int(_lib.mtp_subset_build(_addr(tokens), n_tokens, vocab_size, n, _addr(workspace), workspace_bytes,
                                     _addr(ids_out), _addr(counts_out), _addr(invalid_out), stream))


def mtp_subset_static_max_vocab() -> int:
    return int(_lib.mtp_subset_static_max_vocab())


def mtp_subset_build_static(tokens, n_tokens: int, vocab_size: int, n: int, ids_out, counts_out=None,
                            invalid_out=None, stream=0) -> int:
    return int(_lib.mtp_subset_build_static(_addr(tokens), n_tokens, vocab_size, n, _addr(ids_out),
                                            _addr(counts_out), _addr(invalid_out), stream))


def build_subset(tokens, vocab_size: int, n: int, want_counts: bool = False, stream: int = 0):
    """tokens: device int32 tensor.  Returns dict(ids [n], counts [V] or None, invalid [1]) of device tensors."""
    import torch
    dev = tokens.device
    nbytes = mtp_subset_workspace_bytes(vocab_size)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ids = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    counts = torch.empty(vocab_size, dtype=torch.int32, device=dev) if want_counts else None
    invalid = torch.empty(4, dtype=torch.int32, device=dev)
    st = mtp_subset_build(tokens, tokens.numel(), vocab_size, n, ws, nbytes, ids, counts, invalid, stream)
    if st != MTP_OK:
        raise MTPError(st)
    return {"ids": ids[:n], "counts": counts, "invalid": invalid[:1], "workspace": ws}


def mtp_draft_continue(handle, B: int, K: int, subset_index: int, own_hidden, token_in, k_cache, v_cache, kv_len,
                       forced_tokens, draft_out, logits_out=None, hidden_out=None, stream=0) -> int:
    return int(_lib.mtp_draft_continue(handle, B, K, subset_index, _addr(own_hidden), _addr(token_in), _addr(k_cache),
                                       _addr(v_cache), _addr(kv_len), _addr(forced_tokens), _addr(draft_out),
                                       _addr(logits_out), _addr(hidden_out), stream))


def mtp_draft_extend(handle, B: int, m_max: int, subset_index: int, hidden_in, tokens, ext_len, k_cache, v_cache,
                     kv_len, draft_out, logits_out=None, hidden_out=None, stream=0) -> int:
    return int(_lib.mtp_draft_extend(handle, B, m_max, subset_index, _addr(hidden_in), _addr(tokens), _addr(ext_len),
                                     _addr(k_cache), _addr(v_cache), _addr(kv_len), _addr(draft_out),
                                     _addr(logits_out), _addr(hidden_out), stream))


def mtp_draft_steps(handle, B: int, K: int, subset_index: int, hidden_in, token_in, k_cache, v_cache, kv_len,
                    forced_tokens, draft_out, logits_out, hidden_out, stream: int = 0) -> int:
    return int(_lib.mtp_draft_steps(handle, B, K, subset_index, _addr(hidden_in), _addr(token_in), _addr(k_cache),
                                    _addr(v_cache), _addr(kv_len), _addr(forced_tokens), _addr(draft_out),
                                    _addr(logits_out), _addr(hidden_out), stream or None))


def mtp_accept(handle, B: int, K: int, draft, target, rollback_mode: int, kv_len, accept_len, out_tokens, pending,
               stream: int = 0) -> int:
    return int(_lib.mtp_accept(handle, B, K, _addr(draft), _addr(target), rollback_mode, _addr(kv_len),
                               _addr(accept_len), _addr(out_tokens), _addr(pending), stream or None))


def mtp_poll_error(handle, stream: int = 0) -> int:
    return int(_lib.mtp_poll_error(handle, stream or None))


def mtp_set_timing(handle, mode: int) -> int:
    return int(_lib.mtp_set_timing(handle, mode))


def mtp_last_draft_ms(handle) -> float:
    return float(_lib.mtp_last_draft_ms(handle))


def mtp_set_launch_mode(handle, mode: int) -> int:
    return int(_lib.mtp_set_launch_mode(handle, mode))


def mtp_stream_probe(buffer, nbytes: int, out8, stream=0) -> int:
    return int(_lib.mtp_stream_probe(_addr(buffer), nbytes, _addr(out8), stream))


def mtp_phase_trace_bytes(cfg: mtp_config) -> int:
    return int(_lib.mtp_phase_trace_bytes(C.byref(cfg)))


TRACE_SECTIONS = ["proj", "qkv", "attn", "oproj", "gateup", "down", "lmhead", "unused"]
TRACE_POINTS = ["requested", "released", "staged", "done"]


def mtp_set_phase_trace(handle, device_buffer) -> int:
    return int(_lib.mtp_set_phase_trace(handle, _addr(device_buffer)))


def mtp_draft_destroy(handle) -> None:
    _lib.mtp_draft_destroy(handle)


class MTPError(RuntimeError):
    def __init__(self, status: int):
        super().__init__(f"{STATUS.get(status, status)}: {mtp_status_string(status)}")
        self.status = status


class DraftEngine:
    """Convenience owner of the device buffers of one handle (memory plumbing only).

    weights_bits: name -> numpy uint16 array (bf16 bit patterns); subsets: list of sorted int32 numpy id lists.
    """

    def __init__(self, shape, weights_bits: Dict[str, object], subsets: Sequence[object], max_batch: int,
                 kv_capacity: int, max_draft_steps: int, device: str = "cuda:0", guard_bytes: int = 0):
        import numpy as np
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.shape = shape
        self.cfg = make_config(shape, max_batch, kv_capacity, max_draft_steps)
        # numpy bit patterns are uploaded; tensors already on the device are shared as they are
        self.w = {k: (v if isinstance(v, torch.Tensor) else
                      torch.from_numpy(np.ascontiguousarray(v).view(np.int16)).to(self.device))
                  for k, v in weights_bits.items()}
        self.subsets = [torch.from_numpy(np.ascontiguousarray(s, dtype=np.int32)).to(self.device) for s in subsets]
        nbytes = mtp_workspace_bytes(self.cfg)
        if nbytes == 0:
            raise MTPError(-3)
        # guard_bytes (a multiple of 256): that many bytes of a fixed pattern in front of and behind the workspace, for
        # tests that check that nothing is written outside it (guards_intact)
        self.guard_bytes = guard_bytes
        self._arena = torch.full((nbytes + 2 * guard_bytes,), 0xA5, dtype=torch.uint8, device=self.device)
        self.workspace = self._arena[guard_bytes:guard_bytes + nbytes]
        st, self.handle = mtp_draft_init(self.cfg, self.w, self.subsets, [s.numel() for s in self.subsets],
                                         self.workspace, nbytes)
        if st != MTP_OK:
            raise MTPError(st)

    def guards_intact(self) -> bool:
        g = self.guard_bytes
        return g == 0 or bool((self._arena[:g] == 0xA5).all().item() and (self._arena[-g:] == 0xA5).all().item())

    def subset_size(self, subset_index: int) -> int:
        return self.shape.vocab_size if subset_index < 0 else self.subsets[subset_index].numel()

    def to_device_bits(self, a):
        import numpy as np
        return self.torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(self.device)

    def to_device_i32(self, a):
        import numpy as np
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.device)

    def draft(self, K: int, subset_index: int, hidden_in, token_in, k_cache, v_cache, kv_len, forced=None,
              want_logits: bool = False, want_hidden: bool = False, stream: int = 0):
        """All tensor arguments are device tensors.  Returns dict(draft, logits, hidden) of device tensors."""
        torch = self.torch
        B = token_in.numel()
        n = self.subset_size(subset_index)
        draft = torch.empty((B, K), dtype=torch.int32, device=self.device)
        logits = torch.empty((B, K, n), dtype=torch.float32, device=self.device) if want_logits else None
        hidden = torch.empty((B, K, self.shape.d_model), dtype=torch.float32, device=self.device) if want_hidden \
            else None
        st = mtp_draft_steps(self.handle, B, K, subset_index, hidden_in, token_in, k_cache, v_cache, kv_len, forced,
                             draft, logits, hidden, stream)
        if st != MTP_OK:
            raise MTPError(st)
        return {"draft": draft, "logits": logits, "hidden": hidden}

    def train_loss(self, hidden_in, tokens, K: int, beta: float, stream: int = 0, want_logits: bool = False):
        """Teacher-forced K-step forward and its weighted cross-entropy (see mtp_train_loss).  hidden_in [n][d] bf16
        bits, tokens [n + K + 1]: device tensors.  Returns a device tensor [K + 1]: CE_1 .. CE_K, the loss; with
        want_logits also the last step's logits [n][V] (a view of the call's scratch buffer)."""
        torch = self.torch
        n_pos = hidden_in.shape[0]
        s = self.shape
        nbytes = int(_lib.mtp_train_workspace_bytes(C.byref(self.cfg), n_pos))
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        cache = torch.zeros((2, s.n_kv_heads, self.cfg.kv_capacity, s.head_dim), dtype=torch.int16, device=self.device)
        out = torch.zeros(K + 1 + 3, dtype=torch.float32, device=self.device)
        st = int(_lib.mtp_train_loss(self.handle, n_pos, K, float(beta), _addr(hidden_in), _addr(tokens),
                                     _addr(cache[0]), _addr(cache[1]), _addr(scratch), nbytes, _addr(out), stream))
        if st != MTP_OK:
            raise MTPError(st)
        self._train_keep = (scratch, cache)   # alive until the stream has run the call
        if want_logits:
            return out[:K + 1], scratch[:n_pos * s.vocab_size * 4].view(torch.float32).view(n_pos, s.vocab_size)
        return out[:K + 1]

    def draft_lists(self, K: int, seq_subset, hidden_in, token_in, k_cache, v_cache, kv_len, forced=None,
                    want_logits: bool = False, want_hidden: bool = False, stream: int = 0):
        """Draft steps with one id list per sequence (host list seq_subset).  logits: [B][K][largest list]."""
        torch = self.torch
        B = token_in.numel()
        n_max = max(self.subset_size(int(s)) for s in seq_subset)
        draft = torch.empty((B, K), dtype=torch.int32, device=self.device)
        logits = torch.zeros((B, K, n_max), dtype=torch.float32, device=self.device) if want_logits else None
        hidden = torch.empty((B, K, self.shape.d_model), dtype=torch.float32, device=self.device) if want_hidden \
            else None
        st = mtp_draft_steps_lists(self.handle, B, K, seq_subset, hidden_in, token_in, k_cache, v_cache, kv_len,
                                   forced, draft, logits, hidden, stream)
        if st != MTP_OK:
            raise MTPError(st)
        return {"draft": draft, "logits": logits, "hidden": hidden}

    def draft_continue(self, K: int, subset_index: int, own_hidden, token_in, k_cache, v_cache, kv_len, forced=None,
                       want_logits: bool = False, want_hidden: bool = False, stream: int = 0):
        """Draft steps from the head's own fp32 hidden state [B][d] (see mtp_draft_continue)."""
        torch = self.torch
        B = token_in.numel()
        n = self.subset_size(subset_index)
        draft = torch.empty((B, K), dtype=torch.int32, device=self.device)
        logits = torch.empty((B, K, n), dtype=torch.float32, device=self.device) if want_logits else None
        hidden = torch.empty((B, K, self.shape.d_model), dtype=torch.float32, device=self.device) if want_hidden \
            else None
        st = mtp_draft_continue(self.handle, B, K, subset_index, own_hidden, token_in, k_cache, v_cache, kv_len,
                                forced, draft, logits, hidden, stream)
        if st != MTP_OK:
            raise MTPError(st)
        return {"draft": draft, "logits": logits, "hidden": hidden}

    def extend(self, subset_index: int, hidden_in, tokens, ext_len, k_cache, v_cache, kv_len,
               want_logits: bool = False, want_hidden: bool = False, stream: int = 0):
        """First draft step over a block of new positions.  hidden_in [m_max][B][d] bf16 bits, tokens [m_max][B],
        ext_len [B]: device tensors; kv_len is advanced in place.  Returns dict(draft, logits, hidden)."""
        torch = self.torch
        m_max, B = tokens.shape
        n = self.subset_size(subset_index)
        draft = torch.empty((m_max, B), dtype=torch.int32, device=self.device)
        logits = torch.zeros((m_max, B, n), dtype=torch.float32, device=self.device) if want_logits else None
        hidden = torch.zeros((m_max, B, self.shape.d_model), dtype=torch.float32, device=self.device) \
            if want_hidden else None
        st = mtp_draft_extend(self.handle, B, m_max, subset_index, hidden_in, tokens, ext_len, k_cache, v_cache,
                              kv_len, draft, logits, hidden, stream)
        if st != MTP_OK:
            raise MTPError(st)
        return {"draft": draft, "logits": logits, "hidden": hidden}

    def accept(self, draft, target, kv_len, mode: int = 0, stream: int = 0):
        torch = self.torch
        B, K = draft.shape
        acc = torch.empty(B, dtype=torch.int32, device=self.device)
        out = torch.empty((B, K + 1), dtype=torch.int32, device=self.device)
        pend = torch.empty(B, dtype=torch.int32, device=self.device)
        st = mtp_accept(self.handle, B, K, draft, target, mode, kv_len, acc, out, pend, stream)
        if st != MTP_OK:
            raise MTPError(st)
        return {"accept_len": acc, "out_tokens": out, "pending": pend, "kv_len": kv_len}

    def poll_error(self, stream: int = 0) -> int:
        return mtp_poll_error(self.handle, stream)

    def close(self) -> None:
        if getattr(self, "handle", None) is not None:
            mtp_draft_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
