"""ctypes wrapper around the plain-C oracle (mtp_oracle.c).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, the smoke check and the
benchmark's cpu_baseline leg; never from the product package.  It does not
import the HIP binding and shares nothing with it.

Two builds of the same source: `f32` (the reference precision of this build) and
`f64` (bounds the float build's own rounding error).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mtp_oracle.c")


def lib_path(precision: str) -> str:
    return os.path.join(_HERE, f"libmtp_oracle_{precision}.so")


def build(force: bool = False) -> None:
    """Compile both precisions with gcc (plain -O2: no fast-math, sums stay left to right)."""
    for prec, flag in (("f32", []), ("f64", ["-DORC_F64"])):
        out = lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", *flag, _SRC,
               "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


class _Config(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("kv_capacity", C.c_int32),
                ("recur_pre_norm", C.c_int32)]


_W_FIELDS = ["embed", "lm_head", "g_hnorm", "g_enorm", "g_attn_norm", "g_mlp_norm", "g_final_norm", "w_proj",
             "w_q", "w_k", "w_v", "b_q", "b_k", "b_v", "w_o", "w_gate", "w_up", "w_down"]
_T_FIELDS = ["c", "x", "q", "k", "v", "attn", "x1", "m", "x2"]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_FIELDS]


class _Trace(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _T_FIELDS]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


class Oracle:
    """shape: any object with d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab_size, rms_eps, rope_theta."""

    def __init__(self, shape, weights: Dict[str, np.ndarray], kv_capacity: int, precision: str = "f32",
                 recur_pre_norm: bool = False):
        build()
        self.lib = C.CDLL(lib_path(precision))
        self.real = np.float32 if precision == "f32" else np.float64
        assert self.lib.orc_real_bytes() == np.dtype(self.real).itemsize
        self.shape = shape
        self.cfg = _Config(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                           shape.vocab_size, shape.rms_eps, shape.rope_theta, kv_capacity, int(recur_pre_norm))
        self._keep = {k: _u16(v) for k, v in weights.items()}
        self.w = _Weights(**{n: (_ptr(self._keep[n]) if n in self._keep else None) for n in _W_FIELDS})
        self.lib.orc_round_bf16.restype = C.c_uint16
        self.lib.orc_round_bf16.argtypes = [C.c_float if precision == "f32" else C.c_double]
        self.lib.orc_widen_bf16.restype = C.c_float
        self.lib.orc_widen_bf16.argtypes = [C.c_uint16]

    # -- helpers ---------------------------------------------------------
    @property
    def threads(self) -> int:
        return int(self.lib.orc_num_threads())

    def set_threads(self, n: int) -> None:
        self.lib.orc_set_threads(C.c_int(n))

    def _r(self, a) -> np.ndarray:
        return np.ascontiguousarray(a, dtype=self.real)

    def round_bf16(self, x: float) -> int:
        return int(self.lib.orc_round_bf16(x))

    # -- building blocks ---------------------------------------------------
    def rmsnorm(self, u, g_bits, eps: Optional[float] = None) -> np.ndarray:
        u = self._r(u)
        g = _u16(g_bits)
        out = np.empty_like(u)
        eps = self.shape.rms_eps if eps is None else eps
        self.lib.orc_rmsnorm(_ptr(u), _ptr(g), C.c_int32(u.size), C.c_float(eps), _ptr(out))
        return out

    def linear(self, W_bits, x, bias_bits=None) -> np.ndarray:
        W = _u16(W_bits)
        x = self._r(x)
        n_out, n_in = W.shape
        assert x.size == n_in
        b = None if bias_bits is None else _u16(bias_bits)
        y = np.empty(n_out, dtype=self.real)
        self.lib.orc_linear(_ptr(W), _ptr(b), _ptr(x), C.c_int32(n_out), C.c_int32(n_in), _ptr(y))
        return y

    def rope(self, u, n_heads: int, head_dim: int, pos: int, theta: Optional[float] = None) -> np.ndarray:
        u = self._r(u).copy()
        theta = self.shape.rope_theta if theta is None else theta
        self.lib.orc_rope(_ptr(u), C.c_int32(n_heads), C.c_int32(head_dim), C.c_int32(pos), C.c_float(theta))
        return u

    def attention(self, q, kc_bits, vc_bits, length: int) -> np.ndarray:
        kc, vc = _u16(kc_bits), _u16(vc_bits)
        Hkv, cap, hd = kc.shape
        q = self._r(q)
        Hq = q.size // hd
        out = np.empty(Hq * hd, dtype=self.real)
        rc = self.lib.orc_attention(_ptr(q), _ptr(kc), _ptr(vc), C.c_int32(length), C.c_int32(cap), C.c_int32(Hq),
                                    C.c_int32(Hkv), C.c_int32(hd), _ptr(out))
        if rc:
            raise ValueError(f"orc_attention failed: {rc}")
        return out.reshape(Hq, hd)

    def swiglu(self, w_gate_bits, w_up_bits, y) -> np.ndarray:
        wg, wu = _u16(w_gate_bits), _u16(w_up_bits)
        F, d = wg.shape
        y = self._r(y)
        m = np.empty(F, dtype=self.real)
        self.lib.orc_swiglu(_ptr(wg), _ptr(wu), _ptr(y), C.c_int32(F), C.c_int32(d), _ptr(m))
        return m

    def lm_head(self, W_bits, ids, h):
        """Returns (logits [n], best_index, margin)."""
        W = _u16(W_bits)
        V, d = W.shape
        ids_a = None if ids is None else _i32(ids)
        n = V if ids_a is None else ids_a.size
        h = self._r(h)
        z = np.empty(n, dtype=self.real)
        bi = C.c_int32(0)
        mg = (C.c_float if self.real == np.float32 else C.c_double)(0)
        rc = self.lib.orc_lm_head(_ptr(W), C.c_int32(V), _ptr(ids_a), C.c_int32(n), C.c_int32(d), _ptr(h), _ptr(z),
                                  C.byref(bi), C.byref(mg))
        if rc:
            raise ValueError(f"orc_lm_head failed: {rc}")
        return z, int(bi.value), float(mg.value)

    # -- one step / K steps --------------------------------------------------
    def step(self, h, token: int, kc_bits: np.ndarray, vc_bits: np.ndarray, pos: int, ids, want_logits=True,
             trace: bool = False):
        """One head application for one sequence.  kc_bits/vc_bits [Hkv][cap][hd] are updated in place.
        Returns dict(hhat, logits, draft, margin, [trace arrays])."""
        s = self.shape
        assert kc_bits.dtype == np.uint16 and kc_bits.flags.c_contiguous and vc_bits.flags.c_contiguous
        assert kc_bits.shape == (s.n_kv_heads, self.cfg.kv_capacity, s.head_dim)
        h = self._r(h)
        ids_a = None if ids is None else _i32(ids)
        n = s.vocab_size if ids_a is None else ids_a.size
        hhat = np.empty(s.d_model, dtype=self.real)
        logits = np.empty(n, dtype=self.real) if want_logits else None
        did = C.c_int32(-1)
        mg = (C.c_float if self.real == np.float32 else C.c_double)(0)
        tr_arrays = None
        tr = None
        if trace:
            sizes = {"c": 2 * s.d_model, "x": s.d_model, "q": s.n_q_heads * s.head_dim,
                     "k": s.n_kv_heads * s.head_dim, "v": s.n_kv_heads * s.head_dim,
                     "attn": s.n_q_heads * s.head_dim, "x1": s.d_model, "m": s.d_ffn, "x2": s.d_model}
            tr_arrays = {k: np.empty(v, dtype=self.real) for k, v in sizes.items()}
            tr = _Trace(**{k: _ptr(v) for k, v in tr_arrays.items()})
        rc = self.lib.orc_step(C.byref(self.cfg), C.byref(self.w), _ptr(h), C.c_int32(token), _ptr(kc_bits),
                               _ptr(vc_bits), C.c_int32(pos), _ptr(ids_a), C.c_int32(n), _ptr(hhat), _ptr(logits),
                               C.byref(did), C.byref(mg), C.byref(tr) if tr is not None else None)
        if rc:
            raise ValueError(f"orc_step failed: {rc}")
        out = {"hhat": hhat, "logits": logits, "draft": int(did.value), "margin": float(mg.value)}
        if tr_arrays:
            out.update(tr_arrays)
        return out

    def chain(self, K: int, hidden_in_bits, token_in, k_cache_bits, v_cache_bits, kv_len, ids, forced=None,
              want_logits: bool = True, want_hidden: bool = True):
        """K recursive draft steps for a batch.  Caches [B][Hkv][cap][hd] are updated in place.
        Returns dict(draft [B][K], logits [B][K][n], hidden [B][K][d], margin [B][K])."""
        s = self.shape
        hid = _u16(hidden_in_bits)
        B = hid.shape[0]
        tok = _i32(token_in)
        kvl = _i32(kv_len)
        assert k_cache_bits.dtype == np.uint16 and k_cache_bits.flags.c_contiguous and v_cache_bits.flags.c_contiguous
        assert k_cache_bits.shape[1:] == (s.n_kv_heads, self.cfg.kv_capacity, s.head_dim)
        assert k_cache_bits.shape[0] >= B
        ids_a = None if ids is None else _i32(ids)
        n = s.vocab_size if ids_a is None else ids_a.size
        fr = None if forced is None else _i32(forced).reshape(B, K - 1)
        draft = np.full((B, K), -1, dtype=np.int32)
        logits = np.empty((B, K, n), dtype=self.real) if want_logits else None
        hidden = np.empty((B, K, s.d_model), dtype=self.real) if want_hidden else None
        margin = np.empty((B, K), dtype=self.real)
        rc = self.lib.orc_chain(C.byref(self.cfg), C.byref(self.w), C.c_int32(B), C.c_int32(K), _ptr(hid), _ptr(tok),
                                _ptr(k_cache_bits), _ptr(v_cache_bits), _ptr(kvl), _ptr(fr), _ptr(ids_a),
                                C.c_int32(n), _ptr(draft), _ptr(logits), _ptr(hidden), _ptr(margin))
        if rc:
            raise ValueError(f"orc_chain failed: {rc}")
        return {"draft": draft, "logits": logits, "hidden": hidden, "margin": margin}


    def chain_from_own_hidden(self, K: int, hhat, token: int, kc_bits, vc_bits, pos: int, ids, forced=None):
        """K recursive steps of ONE sequence that start from the head's own output hidden state (Sec. 2.3: from the
        second step on): single steps fed back by hand.  forced [K-1]: tokens fed at the later steps instead of the
        previous draft.  Returns dict(draft [K], logits [K][n], hidden [K][d], margin [K])."""
        h, tok = self._r(hhat), int(token)
        out = {"draft": [], "logits": [], "hidden": [], "margin": []}
        for k in range(K):
            r = self.step(h, tok, kc_bits, vc_bits, pos + k, ids)
            for key, name in (("draft", "draft"), ("logits", "logits"), ("hidden", "hhat"), ("margin", "margin")):
                out[key].append(r[name])
            h = r["hhat"]
            tok = int(forced[k]) if (forced is not None and k + 1 < K) else r["draft"]
        return {k: np.array(v) for k, v in out.items()}

    def extend(self, hidden_in_bits, tokens, ext_len, k_cache_bits, v_cache_bits, kv_len, ids,
               want_logits: bool = True, want_hidden: bool = True):
        """First draft step over several new positions (Sec. 2.3, "Drafting phase").
        hidden_in_bits [m_max][B][d] bf16, tokens [m_max][B], ext_len [B].  Caches are updated in place.
        Returns dict(draft [m_max][B], logits [m_max][B][n], hidden [m_max][B][d], margin [m_max][B],
        kv_len [B] (new), overflow bool)."""
        s = self.shape
        hid = _u16(hidden_in_bits)
        m_max, B = hid.shape[0], hid.shape[1]
        tok = _i32(tokens).reshape(m_max, B)
        el = _i32(ext_len)
        kvl = _i32(kv_len).copy()
        assert k_cache_bits.dtype == np.uint16 and k_cache_bits.flags.c_contiguous and v_cache_bits.flags.c_contiguous
        assert k_cache_bits.shape[1:] == (s.n_kv_heads, self.cfg.kv_capacity, s.head_dim)
        ids_a = None if ids is None else _i32(ids)
        n = s.vocab_size if ids_a is None else ids_a.size
        draft = np.full((m_max, B), -1, dtype=np.int32)
        logits = np.zeros((m_max, B, n), dtype=self.real) if want_logits else None
        hidden = np.zeros((m_max, B, s.d_model), dtype=self.real) if want_hidden else None
        margin = np.zeros((m_max, B), dtype=self.real)
        rc = self.lib.orc_extend(C.byref(self.cfg), C.byref(self.w), C.c_int32(B), C.c_int32(m_max), _ptr(hid),
                                 _ptr(tok), _ptr(el), _ptr(k_cache_bits), _ptr(v_cache_bits), _ptr(kvl), _ptr(ids_a),
                                 C.c_int32(n), _ptr(draft), _ptr(logits), _ptr(hidden), _ptr(margin))
        if rc not in (0, 1):
            raise ValueError(f"orc_extend failed: {rc}")
        return {"draft": draft, "logits": logits, "hidden": hidden, "margin": margin, "kv_len": kvl,
                "overflow": rc == 1}


def loss_weights(K: int, beta: float) -> np.ndarray:
    """Eq. (2): alpha_k = beta^(k-1) / sum_j beta^(j-1), k = 1..K."""
    w = np.power(float(beta), np.arange(K, dtype=np.float64))
    return w / w.sum()


def train_loss(orc: "Oracle", hidden_in_bits, tokens, K: int, beta: float):
    """Teacher-forced K-step forward of the shared head over all positions of one sequence and the weighted
    cross-entropy of Eq. (1) (Sec. 2.1 "Training Mechanism" / "Training Objective"), forward only.
      hidden_in_bits [n_pos][d] bf16: the main model's hidden states h_1 .. h_n (positions i = 1 .. n = T - K)
      tokens [n_pos + K + 1]: t_1 .. t_{n+K+1}
    Step k at position i consumes (h^{k-1}_i, embedding of t_{i+k}) and is scored against t_{i+k+1}; h^0 is the main
    model's state, h^k the head's own output; inside a step a position attends the step's own keys of positions <= i
    (a fresh cache per step, slot = position index; rotary attention only sees position differences).  CE_k is the
    mean over the n positions of logsumexp(z) - z[label] over the FULL vocabulary, in float64 from the step's logits.
    Returns dict(ce [K], loss, alpha [K], logits [K][n][V], hidden [K][n][d])."""
    s = orc.shape
    hid = _u16(hidden_in_bits)
    n = hid.shape[0]
    tok = _i32(tokens)
    assert tok.shape == (n + K + 1,)
    cap = orc.cfg.kv_capacity
    assert n <= cap
    h = bf16_to_real(hid, orc.real)
    ce = np.zeros(K)
    all_logits, all_hidden = [], []
    for k in range(1, K + 1):
        kc = np.zeros((s.n_kv_heads, cap, s.head_dim), dtype=np.uint16)
        vc = np.zeros_like(kc)
        logits = np.empty((n, s.vocab_size), dtype=orc.real)
        nxt = np.empty((n, s.d_model), dtype=orc.real)
        for i in range(n):                       # position i + 1 of the text
            r = orc.step(h[i], int(tok[i + k]), kc, vc, i, None)
            logits[i], nxt[i] = r["logits"], r["hhat"]
        z = logits.astype(np.float64)
        m = z.max(axis=1)
        lse = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
        ce[k - 1] = float((lse - z[np.arange(n), tok[k + 1:k + 1 + n]]).mean())
        all_logits.append(logits)
        all_hidden.append(nxt)
        h = nxt
    alpha = loss_weights(K, beta)
    return {"ce": ce, "loss": float((alpha * ce).sum()), "alpha": alpha, "logits": np.array(all_logits),
            "hidden": np.array(all_hidden)}


def bf16_to_real(bits: np.ndarray, real) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(real)


def build_subset(tokens, vocab_size: int, n: int):
    """The high-frequency id list of Sec. 2.2 (which takes it from statistics over a corpus) from a token stream:
    occurrence counts per id, the n ids with the largest counts (equal counts: the lower id first), returned in
    ascending id order - the format the output head of Eq. (3) is gathered with.  Ids outside [0, vocab_size) are
    skipped and counted.  Returns dict(counts [V] int64, ids [n] int32, invalid int)."""
    t = np.asarray(tokens, dtype=np.int64).ravel()
    ok = (t >= 0) & (t < vocab_size)
    counts = np.bincount(t[ok], minlength=vocab_size)
    if not 0 <= n <= vocab_size:
        raise ValueError("n outside 0 .. vocab_size")
    order = np.lexsort((np.arange(vocab_size), -counts))      # by count descending, then id ascending
    return {"counts": counts, "ids": np.sort(order[:n]).astype(np.int32), "invalid": int((~ok).sum())}


def accept(draft, target, kv_len, mode: int = 0, precision: str = "f32"):
    """Returns dict(accept_len [B], out_tokens [B][K+1], kv_len [B] (new), pending [B])."""
    build()
    lib = C.CDLL(lib_path(precision))
    dr = _i32(draft)
    B, K = dr.shape
    tg = _i32(target).reshape(B, K + 1)
    kvl = _i32(kv_len).copy()
    acc = np.empty(B, dtype=np.int32)
    out = np.empty((B, K + 1), dtype=np.int32)
    pend = np.empty(B, dtype=np.int32)
    lib.orc_accept(C.c_int32(B), C.c_int32(K), _ptr(dr), _ptr(tg), C.c_int32(mode), _ptr(kvl), _ptr(acc), _ptr(out),
                   _ptr(pend))
    return {"accept_len": acc, "out_tokens": out, "kv_len": kvl, "pending": pend}
