"""Seeded synthetic inputs for the FastMTP draft path.

This module only draws random numbers and lays them out in the interface
formats (bf16 bit patterns as uint16, int32 ids).  It contains none of the
method's arithmetic: no norm, no projection, no attention, no argmax.  Both the
CPU oracle and the HIP library are fed the arrays produced here, bit for bit.

The paper (Sec. 3.1, "Model Configuration") evaluates on MiMo-7B-RL with a
fine-tuned MTP head and on public benchmark prompts; none of that is available
offline, so seeded tensors of the same shapes stand in for them:

* matrices, biases, embedding table and output head  ~ N(0, 0.02)
* RMSNorm gains                                       ~ 1 + N(0, 0.02)
* target hidden state, prior keys and values          ~ N(0, 1)
* compressed vocabularies: ids drawn without replacement, weight 1/(id+1)
  (a long-tailed frequency profile as described in Sec. 2.2), sorted ascending;
  nested sizes come from one ranking, like a frequency-ranked list.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence

import numpy as np

BASE_SEED = 250918362
_CHUNK = 1 << 22  # elements drawn per independent stream
_DIRECT_CACHE_ELEMS = 1 << 28  # KV caches up to this size are drawn element by element
_POOL_ELEMS = 1 << 26


@dataclasses.dataclass(frozen=True)
class HeadShape:
    """Shape of one MTP head (Sec. 2.1 "Architecture Design", Sec. 3.1)."""

    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab_size: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


TINY = HeadShape(256, 4, 2, 64, 688, 4096)
SEVEN_B = HeadShape(4096, 32, 8, 128, 11008, 151680)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark configuration: a head shape plus the drafting scenario."""

    name: str
    index: int  # enters the seed
    shape: HeadShape
    batch: int
    ctx_lo: int
    ctx_hi: int  # inclusive; ctx_lo == ctx_hi -> fixed context
    subset_sizes: Sequence[int]  # nested compressed vocabularies
    draft_steps: int
    accept_prob: float
    zipf_subset: bool = True


WORKLOADS: Dict[str, Workload] = {
    "c1_tiny": Workload("c1_tiny", 1, TINY, 1, 128, 128, (1024,), 3, 0.5, zipf_subset=False),
    "c2_7b_b1": Workload("c2_7b_b1", 2, SEVEN_B, 1, 2048, 2048, (32768,), 3, 0.5),
    "c3_7b_b16": Workload("c3_7b_b16", 3, SEVEN_B, 16, 512, 4096, (32768,), 3, 0.8),
    "c4_7b_vocab": Workload("c4_7b_vocab", 4, SEVEN_B, 1, 8192, 8192, (16384, 32768, 65536), 3, 0.5),
    "c5_7b_b64": Workload("c5_7b_b64", 5, SEVEN_B, 64, 8192, 32768, (32768,), 5, 0.7),
}


def _rng(config_index: int, stream_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config_index + stream_id))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(config_index: int, stream_id: int, shape, mean: float, std: float,
                threads: int = 8) -> np.ndarray:
    """bf16 bits of mean + std * N(0,1).  The tensor is cut into fixed-size chunks,
    each drawn from its own child stream, so the bits do not depend on `threads`."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    n_chunks = (n + _CHUNK - 1) // _CHUNK
    children = np.random.SeedSequence(BASE_SEED + 1000 * config_index + stream_id).spawn(n_chunks)

    def fill(i: int) -> None:
        lo, hi = i * _CHUNK, min(n, (i + 1) * _CHUNK)
        g = np.random.Generator(np.random.PCG64(children[i]))
        v = g.standard_normal(hi - lo, dtype=np.float32)
        v *= np.float32(std)
        v += np.float32(mean)
        out[lo:hi] = f32_to_bf16_bits(v)

    if n_chunks == 1 or threads <= 1:
        for i in range(n_chunks):
            fill(i)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


# stream ids -----------------------------------------------------------------
_W_STREAMS = ["embed", "lm_head", "g_hnorm", "g_enorm", "g_attn_norm", "g_mlp_norm", "g_final_norm",
              "w_proj", "w_q", "w_k", "w_v", "b_q", "b_k", "b_v", "w_o", "w_gate", "w_up", "w_down"]
_S_HIDDEN, _S_TOKEN, _S_CTX, _S_KCACHE, _S_VCACHE, _S_SUBSET, _S_TARGET = 100, 101, 102, 103, 104, 105, 106


def weight_shapes(s: HeadShape) -> Dict[str, tuple]:
    """Row-major [out][in] shapes of every tensor of the head."""
    d = s.d_model
    return {
        "embed": (s.vocab_size, d), "lm_head": (s.vocab_size, d),
        "g_hnorm": (d,), "g_enorm": (d,), "g_attn_norm": (d,), "g_mlp_norm": (d,), "g_final_norm": (d,),
        "w_proj": (d, 2 * d),
        "w_q": (s.q_dim, d), "w_k": (s.kv_dim, d), "w_v": (s.kv_dim, d),
        "b_q": (s.q_dim,), "b_k": (s.kv_dim,), "b_v": (s.kv_dim,),
        "w_o": (d, s.q_dim),
        "w_gate": (s.d_ffn, d), "w_up": (s.d_ffn, d), "w_down": (d, s.d_ffn),
    }


def make_weights(wl: Workload, with_bias: bool = True, threads: int = 8,
                 seed_index: Optional[int] = None) -> Dict[str, np.ndarray]:
    """All tensors of the head as bf16 bit patterns (uint16)."""
    idx = wl.index if seed_index is None else seed_index
    out: Dict[str, np.ndarray] = {}
    for sid, (name, shp) in enumerate(weight_shapes(wl.shape).items()):
        assert _W_STREAMS[sid] == name
        if name.startswith("b_") and not with_bias:
            continue
        mean = 1.0 if name.startswith("g_") else 0.0
        out[name] = normal_bf16(idx, sid, shp, mean, 0.02, threads)
    return out


def head_param_count(s: HeadShape) -> int:
    """Trainable parameters of the MTP head: everything but the shared embedding/output head."""
    return sum(int(np.prod(v)) for k, v in weight_shapes(s).items() if k not in ("embed", "lm_head"))


def make_context_lengths(wl: Workload) -> np.ndarray:
    if wl.ctx_lo == wl.ctx_hi:
        return np.full(wl.batch, wl.ctx_lo, dtype=np.int32)
    return _rng(wl.index, _S_CTX).integers(wl.ctx_lo, wl.ctx_hi + 1, size=wl.batch).astype(np.int32)


def kv_capacity_for(wl: Workload, ctx: np.ndarray) -> int:
    return int(-(-(int(ctx.max()) + wl.draft_steps) // 64) * 64)


def make_activations(wl: Workload, ctx: Optional[np.ndarray] = None, threads: int = 8,
                     capacity: Optional[int] = None) -> Dict[str, np.ndarray]:
    """hidden_in [B][d] bf16, token_in [B], kv_len [B], k_cache/v_cache [B][Hkv][cap][hd] bf16.
    Cache slots at or beyond kv_len[b] are zero."""
    s = wl.shape
    if ctx is None:
        ctx = make_context_lengths(wl)
    ctx = np.asarray(ctx, dtype=np.int32)
    B = len(ctx)
    cap = capacity if capacity is not None else kv_capacity_for(wl, ctx)
    hidden = normal_bf16(wl.index, _S_HIDDEN, (B, s.d_model), 0.0, 1.0, threads)
    token = _rng(wl.index, _S_TOKEN).integers(0, s.vocab_size, size=B).astype(np.int32)
    shape = (B, s.n_kv_heads, cap, s.head_dim)
    if int(np.prod(shape)) <= _DIRECT_CACHE_ELEMS:
        kc = normal_bf16(wl.index, _S_KCACHE, shape, 0.0, 1.0, threads)
        vc = normal_bf16(wl.index, _S_VCACHE, shape, 0.0, 1.0, threads)
        for b in range(B):
            kc[b, :, ctx[b]:, :] = 0
            vc[b, :, ctx[b]:, :] = 0
    else:
        # very large caches: every (sequence, KV head) stream is a window, at a seeded offset, into one pool of
        # N(0,1) draws; within a stream the entries are still independent
        pool_k = normal_bf16(wl.index, _S_KCACHE, (_POOL_ELEMS,), 0.0, 1.0, threads)
        pool_v = normal_bf16(wl.index, _S_VCACHE, (_POOL_ELEMS,), 0.0, 1.0, threads)
        offs = _rng(wl.index, _S_KCACHE + 50).integers(0, (_POOL_ELEMS - cap * s.head_dim) // s.head_dim,
                                                       size=(2, B, s.n_kv_heads)) * s.head_dim
        kc = np.zeros(shape, dtype=np.uint16)
        vc = np.zeros(shape, dtype=np.uint16)
        for b in range(B):
            nel = int(ctx[b]) * s.head_dim
            for g in range(s.n_kv_heads):
                kc[b, g].reshape(-1)[:nel] = pool_k[offs[0, b, g]:offs[0, b, g] + nel]
                vc[b, g].reshape(-1)[:nel] = pool_v[offs[1, b, g]:offs[1, b, g] + nel]
    return {"hidden_in": hidden, "token_in": token, "kv_len": ctx.copy(), "k_cache": kc, "v_cache": vc,
            "kv_capacity": cap}


def make_subsets(wl: Workload) -> List[np.ndarray]:
    """Nested sorted-unique id lists, one per entry of wl.subset_sizes."""
    V = wl.shape.vocab_size
    g = _rng(wl.index, _S_SUBSET)
    u = g.random(V)
    if wl.zipf_subset:
        # weighted sampling without replacement by exponent keys: key = u**(1/w), w = 1/(id+1)
        key = np.log(np.maximum(u, 1e-300)) * (np.arange(V, dtype=np.float64) + 1.0)
    else:
        key = u
    order = np.argsort(-key, kind="stable")
    return [np.sort(order[:n]).astype(np.int32) for n in wl.subset_sizes]


def make_token_stream(vocab_size: int, n_tokens: int, seed: int, exponent: float = 1.1,
                      invalid_every: int = 0) -> np.ndarray:
    """Stand-in for a tokenised corpus (the frequency statistics behind the high-frequency lists of Sec. 2.2):
    n_tokens ids drawn independently with P(rank r) ~ 1/(r+1)^exponent, ranks mapped to ids by a seeded
    permutation, so frequent ids are scattered over the vocabulary.  invalid_every > 0 plants an out-of-range id
    (-1 or vocab_size, alternating) at every invalid_every-th position."""
    g = np.random.Generator(np.random.PCG64(BASE_SEED + 77000 + seed))
    w = 1.0 / np.power(np.arange(vocab_size, dtype=np.float64) + 1.0, exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    perm = g.permutation(vocab_size).astype(np.int32)
    out = np.empty(n_tokens, dtype=np.int32)
    step = 1 << 22
    for lo in range(0, n_tokens, step):
        hi = min(n_tokens, lo + step)
        r = np.searchsorted(cdf, g.random(hi - lo), side="right")
        out[lo:hi] = perm[np.minimum(r, vocab_size - 1)]
    if invalid_every > 0:
        idx = np.arange(invalid_every - 1, n_tokens, invalid_every)
        out[idx] = np.where(np.arange(len(idx)) % 2 == 0, -1, vocab_size).astype(np.int32)
    return out


def make_targets(wl: Workload, drafts: np.ndarray, accept_prob: Optional[float] = None,
                 salt: int = 0) -> np.ndarray:
    """Stand-in for the target model's greedy tokens g_1..g_{K+1} (Sec. 2.3, verification):
    position j agrees with the draft with probability accept_prob until the first miss;
    after the first miss, and at position K+1, tokens are uniform."""
    p = wl.accept_prob if accept_prob is None else accept_prob
    V = wl.shape.vocab_size
    drafts = np.asarray(drafts, dtype=np.int64)
    B, K = drafts.shape
    g = _rng(wl.index, _S_TARGET + salt)
    hit = g.random((B, K)) < p
    shift = g.integers(1, V, size=(B, K))
    uni = g.integers(0, V, size=(B, K + 1))
    tgt = np.empty((B, K + 1), dtype=np.int64)
    for b in range(B):
        missed = False
        for j in range(K):
            if missed:
                tgt[b, j] = uni[b, j]
            elif hit[b, j]:
                tgt[b, j] = drafts[b, j]
            else:
                tgt[b, j] = (drafts[b, j] + shift[b, j]) % V
                missed = True
        tgt[b, K] = uni[b, K]
    return tgt.astype(np.int32)
