"""Pins of the CPU oracle against things other than itself: library routines (torch CPU ops and the
Hugging Face Qwen2 decoder layer, both in float64), closed forms, invariants, brute force and the few values the
paper prints.  All run without a GPU."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as orc_mod
from oracle.oracle import Oracle
from paper_2509_18362_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def widen(bits):
    return torch.from_numpy(synth.bf16_bits_to_f32(bits)).double()


def rand_bits(rng, shape, std=1.0, mean=0.0):
    return synth.f32_to_bf16_bits((rng.standard_normal(shape) * std + mean).astype(np.float32))


@pytest.fixture(scope="module", params=["f32", "f64"])
def orc(request, tiny):
    return Oracle(tiny["shape"], tiny["w"], tiny["act"]["kv_capacity"], request.param)


def tol(o, t32, t64):
    return t32 if o.real == np.float32 else t64


# ---------------------------------------------------------------- bf16 rounding
def test_bf16_rounding_matches_torch(orc):
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 3,
                         np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38, 1e-40])])
    # exact ties: 1 + 2^-8 (rounds to even = 1.0), 1 + 3*2^-8 (rounds up to 1 + 2^-6)
    for x in xs:
        want = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).item() & 0xFFFF
        assert orc.round_bf16(float(x)) == want, x


def test_bf16_rounding_f64_no_double_rounding():
    o = Oracle(synth.TINY, {}, 8, "f64")
    # just above the tie 1 + 2^-8 by less than a float ulp: float conversion lands on the tie, true value is above
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert o.round_bf16(x) == 0x3F81
    x = 1.0 + 2.0 ** -8 - 2.0 ** -40
    assert o.round_bf16(x) == 0x3F80


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_vs_library(orc):
    rng = np.random.default_rng(2)
    d = 96
    u = rng.standard_normal(d) * 2.5
    g = rand_bits(rng, d, 0.1, 1.0)
    got = orc.rmsnorm(u, g, eps=1e-6)
    want = F.rms_norm(torch.from_numpy(u.astype(orc.real)).double(), (d,), widen(g), eps=1e-6).numpy()
    np.testing.assert_allclose(got, want, rtol=tol(orc, 2e-6, 1e-13))


def test_rmsnorm_closed_forms(orc):
    d, c, eps = 64, -3.0, 1e-6
    g = rand_bits(np.random.default_rng(3), d, 0.1, 1.0)
    got = orc.rmsnorm(np.full(d, c), g, eps=eps)
    want = synth.bf16_bits_to_f32(g).astype(np.float64) * (np.sign(c) / math.sqrt(1 + eps / c ** 2))
    np.testing.assert_allclose(got, want, rtol=tol(orc, 1e-6, 1e-13))
    # ||out/g||^2 = d / (1 + eps/ms)
    u = np.random.default_rng(4).standard_normal(d)
    ones = synth.f32_to_bf16_bits(np.ones(d, np.float32))
    out = orc.rmsnorm(u, ones, eps=eps).astype(np.float64)
    ms = float(np.mean(u.astype(orc.real).astype(np.float64) ** 2))
    assert abs(np.sum(out ** 2) - d / (1 + eps / ms)) < tol(orc, 1e-4, 1e-10)
    # a large eps matters: eps is inside the square root, added to the mean square
    out = orc.rmsnorm(np.ones(d), ones, eps=3.0).astype(np.float64)
    np.testing.assert_allclose(out, 0.5, rtol=1e-6)


# ---------------------------------------------------------------- linear
def test_linear_vs_library(orc):
    rng = np.random.default_rng(5)
    W = rand_bits(rng, (37, 83), 0.05)
    b = rand_bits(rng, 37, 0.05)
    x = rng.standard_normal(83).astype(orc.real)
    want = F.linear(torch.from_numpy(x).double(), widen(W), widen(b)).numpy()
    np.testing.assert_allclose(orc.linear(W, x, b), want, atol=tol(orc, 2e-6, 1e-13))
    want = F.linear(torch.from_numpy(x).double(), widen(W)).numpy()
    np.testing.assert_allclose(orc.linear(W, x), want, atol=tol(orc, 2e-6, 1e-13))


# ---------------------------------------------------------------- RoPE
def test_rope_known_values(orc):
    # one pair, frequency theta^0 = 1: (1, 0) turns by `pos` radians, counter-clockwise
    out = orc.rope(np.array([1.0, 0.0]), 1, 2, 3, theta=10000.0)
    np.testing.assert_allclose(out, [math.cos(3.0), math.sin(3.0)], atol=1e-6)
    # head_dim 4: pairs are (0,2) and (1,3); second pair turns at theta^(-2/4) = 1/100
    out = orc.rope(np.array([0.0, 1.0, 0.0, 0.0]), 1, 4, 50, theta=10000.0)
    np.testing.assert_allclose(out, [0.0, math.cos(0.5), 0.0, math.sin(0.5)], atol=1e-6)
    out = orc.rope(np.array([0.0, 0.0, 1.0, 0.0]), 1, 4, 2, theta=10000.0)
    np.testing.assert_allclose(out, [-math.sin(2.0), 0.0, math.cos(2.0), 0.0], atol=1e-6)


def test_rope_vs_complex_multiplication(orc):
    rng = np.random.default_rng(6)
    H, hd, pos, theta = 3, 64, 2049, 1e6
    u = rng.standard_normal((H, hd)).astype(orc.real)
    z = u[:, :hd // 2].astype(np.float64) + 1j * u[:, hd // 2:].astype(np.float64)
    w = np.exp(1j * pos * theta ** (-np.arange(hd // 2) * 2.0 / hd))
    zz = z * w[None, :]
    want = np.concatenate([zz.real, zz.imag], axis=1)
    got = orc.rope(u.reshape(-1), H, hd, pos, theta).reshape(H, hd)
    np.testing.assert_allclose(got, want, atol=tol(orc, 2e-6, 1e-12))


def test_rope_invariants(orc):
    rng = np.random.default_rng(7)
    hd = 64
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    np.testing.assert_array_equal(orc.rope(q, 1, hd, 0), q.astype(orc.real))  # position 0 is the identity
    r = orc.rope(q, 1, hd, 777).astype(np.float64)
    assert abs(np.dot(r, r) - np.dot(q.astype(orc.real).astype(np.float64), q.astype(orc.real).astype(np.float64))) < tol(orc, 1e-4, 1e-10)
    # <R_p q, R_t k> depends only on p - t
    dots = [float(np.dot(orc.rope(q, 1, hd, p).astype(np.float64), orc.rope(k, 1, hd, t).astype(np.float64)))
            for p, t in [(10, 3), (107, 100), (1007, 1000)]]
    assert max(dots) - min(dots) < tol(orc, 2e-4, 1e-9)


# ---------------------------------------------------------------- attention
def _sdpa(q, kc, vc, length, group):
    K = widen(kc)[:, :length].repeat_interleave(group, dim=0)
    V = widen(vc)[:, :length].repeat_interleave(group, dim=0)
    qq = torch.from_numpy(np.asarray(q, dtype=np.float64)).reshape(-1, 1, K.shape[-1])
    return F.scaled_dot_product_attention(qq.unsqueeze(0), K.unsqueeze(0), V.unsqueeze(0)).squeeze(0).squeeze(1).numpy()


def test_attention_vs_library(orc):
    rng = np.random.default_rng(8)
    Hq, Hkv, hd, cap, length = 6, 2, 32, 50, 41
    kc, vc = rand_bits(rng, (Hkv, cap, hd)), rand_bits(rng, (Hkv, cap, hd))
    q = (rng.standard_normal((Hq, hd)) * 2).astype(orc.real)
    got = orc.attention(q, kc, vc, length)
    np.testing.assert_allclose(got, _sdpa(q, kc, vc, length, Hq // Hkv), atol=tol(orc, 3e-6, 1e-13))


def test_attention_special_cases(orc):
    rng = np.random.default_rng(9)
    Hq, Hkv, hd, cap = 4, 2, 16, 12
    vc = rand_bits(rng, (Hkv, cap, hd))
    q = rng.standard_normal((Hq, hd)).astype(orc.real)
    # all keys equal: uniform weights, output = mean of the first `length` values
    kc = np.broadcast_to(rand_bits(rng, (Hkv, 1, hd)), (Hkv, cap, hd)).copy()
    got = orc.attention(q, kc, vc, 9)
    want = widen(vc)[:, :9].mean(dim=1).repeat_interleave(2, dim=0).numpy()
    np.testing.assert_allclose(got, want, atol=tol(orc, 1e-6, 1e-13))
    # one key aligned with q and huge: output = that value row
    kc = rand_bits(rng, (Hkv, cap, hd), 0.01)
    kc[0, 5] = synth.f32_to_bf16_bits((q[0] * 200).astype(np.float32))
    got = orc.attention(q, kc, vc, 9)
    np.testing.assert_allclose(got[0], widen(vc)[0, 5].numpy(), atol=1e-6)
    # length 1: output = the single value row, whatever q is
    got = orc.attention(q, kc, vc, 1)
    np.testing.assert_array_equal(got, widen(vc)[:, 0].repeat_interleave(2, dim=0).numpy().astype(orc.real))
    # grouped queries: heads 0,1 read KV head 0; heads 2,3 read KV head 1
    kc = rand_bits(rng, (Hkv, cap, hd))
    qs = np.tile(q[0], (Hq, 1))
    got = orc.attention(qs, kc, vc, 12)
    np.testing.assert_array_equal(got[0], got[1])
    np.testing.assert_array_equal(got[2], got[3])
    assert np.abs(got[0] - got[2]).max() > 1e-3


# ---------------------------------------------------------------- SwiGLU
def test_swiglu_vs_library(orc):
    rng = np.random.default_rng(10)
    Fd, d = 45, 70
    wg, wu = rand_bits(rng, (Fd, d), 0.2), rand_bits(rng, (Fd, d), 0.2)
    y = rng.standard_normal(d).astype(orc.real)
    yt = torch.from_numpy(y).double()
    want = (F.silu(F.linear(yt, widen(wg))) * F.linear(yt, widen(wu))).numpy()
    np.testing.assert_allclose(orc.swiglu(wg, wu, y), want, atol=tol(orc, 3e-6, 1e-13))
    zero = np.zeros((Fd, d), np.uint16)
    np.testing.assert_array_equal(orc.swiglu(zero, wu, y), 0)


# ---------------------------------------------------------------- compressed LM head, Eq. (3)
def test_lm_head_identity_subset_is_full_head(orc, tiny):
    W = tiny["w"]["lm_head"]
    V, d = W.shape
    h = np.random.default_rng(11).standard_normal(d).astype(orc.real)
    z_full, bi_full, mg_full = orc.lm_head(W, None, h)
    z_id, bi_id, mg_id = orc.lm_head(W, np.arange(V, dtype=np.int32), h)
    np.testing.assert_array_equal(z_full, z_id)
    assert (bi_full, mg_full) == (bi_id, mg_id)
    # and the full head is the library's dense product
    want = F.linear(torch.from_numpy(h).double(), widen(W)).numpy()
    np.testing.assert_allclose(z_full, want, atol=tol(orc, 3e-6, 1e-12))
    assert bi_full == int(np.argmax(z_full))


def test_lm_head_subset_rows_argmax_margin(orc, tiny):
    W = tiny["w"]["lm_head"]
    V, d = W.shape
    ids = tiny["ids"]
    assert np.all(np.diff(ids) > 0) and ids[0] >= 0 and ids[-1] < V
    h = np.random.default_rng(12).standard_normal(d).astype(orc.real)
    z_full, _, _ = orc.lm_head(W, None, h)
    z, bi, mg = orc.lm_head(W, ids, h)
    np.testing.assert_array_equal(z, z_full[ids])  # row i of the compressed head is row ids[i] of W
    masked = np.full(V, -np.inf)
    masked[ids] = z_full[ids]
    assert ids[bi] == int(np.argmax(masked))  # brute force over the full vocabulary, restricted to the subset
    top2 = np.sort(z.astype(np.float64))[-2:]
    assert abs(mg - (top2[1] - top2[0])) <= tol(orc, 1e-6, 1e-14)


def test_lm_head_ties_pick_lowest_index(orc):
    rng = np.random.default_rng(13)
    d = 32
    W = rand_bits(rng, (10, d), 0.1)
    h = rng.standard_normal(d).astype(orc.real)
    z, _, _ = orc.lm_head(W, None, h)
    best = int(np.argmax(z))
    W2 = np.concatenate([W, W[best:best + 1]], axis=0)  # duplicate of the winning row at a higher id
    ids = np.array([i for i in range(11)], dtype=np.int32)
    _, bi, mg = orc.lm_head(W2, ids, h)
    assert bi == best and mg == 0.0
    _, bi, _ = orc.lm_head(W2, np.array([3 if best != 3 else 4, best, 10], dtype=np.int32), h)
    assert bi == 1
    with pytest.raises(ValueError):
        orc.lm_head(W, np.array([0, 10], dtype=np.int32), h)  # id outside the vocabulary


# ---------------------------------------------------------------- whole step vs library decoder layer
def _hf_layer(shape, w):
    from transformers.models.qwen2 import modeling_qwen2 as m
    cfg = m.Qwen2Config(hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                        num_attention_heads=shape.n_q_heads, num_key_value_heads=shape.n_kv_heads,
                        num_hidden_layers=1, vocab_size=shape.vocab_size, rms_norm_eps=shape.rms_eps,
                        rope_theta=shape.rope_theta, max_position_embeddings=1 << 16, attn_implementation="eager")
    layer = m.Qwen2DecoderLayer(cfg, 0).double().eval()
    sd = {"self_attn.q_proj.weight": "w_q", "self_attn.q_proj.bias": "b_q", "self_attn.k_proj.weight": "w_k",
          "self_attn.k_proj.bias": "b_k", "self_attn.v_proj.weight": "w_v", "self_attn.v_proj.bias": "b_v",
          "self_attn.o_proj.weight": "w_o", "mlp.gate_proj.weight": "w_gate", "mlp.up_proj.weight": "w_up",
          "mlp.down_proj.weight": "w_down", "input_layernorm.weight": "g_attn_norm",
          "post_attention_layernorm.weight": "g_mlp_norm"}
    layer.load_state_dict({k: widen(w[v]) for k, v in sd.items()}, strict=True)
    rot = m.Qwen2RotaryEmbedding(cfg).double()
    return m, cfg, layer, rot


def test_step_vs_hf_qwen2_decoder_layer(orc, tiny):
    """The decoder layer inside the head (pre-norm GQA attention with q/k/v biases and half-split rotary pairs,
    pre-norm SwiGLU MLP, two residuals) against the Hugging Face Qwen2 layer in float64, fed the same prior keys
    and values.  The library layer does not round the new key/value to bf16, hence the loose outer tolerance; the
    inner comparison repeats the attention with the library's own pieces on the rounded cache."""
    from transformers.cache_utils import DynamicCache
    s, w, act = tiny["shape"], tiny["w"], tiny["act"]
    m, cfg, layer, rot = _hf_layer(s, w)
    L = int(act["kv_len"][0])
    kc, vc = act["k_cache"][0].copy(), act["v_cache"][0].copy()
    h = synth.bf16_bits_to_f32(act["hidden_in"][0]).astype(orc.real)
    token = int(act["token_in"][0])
    res = orc.step(h, token, kc, vc, L, tiny["ids"], trace=True)

    x = torch.from_numpy(res["x"].astype(np.float64)).reshape(1, 1, -1)
    pos = torch.tensor([[L]])
    cos, sin = rot(x, pos)
    cache = DynamicCache(config=cfg)
    cache.update(widen(act["k_cache"])[0:1, :, :L], widen(act["v_cache"])[0:1, :, :L], 0)
    with torch.no_grad():
        out = layer(x, attention_mask=None, position_ids=pos, past_key_values=cache, use_cache=True,
                    position_embeddings=(cos, sin))
        out = out[0] if isinstance(out, tuple) else out
        x2_lib = out.reshape(-1).numpy()
        scale = float(np.abs(x2_lib).max())
        assert np.abs(res["x2"] - x2_lib).max() < 2e-3 * scale

        # piecewise, with the library's modules, on the cache as stored (new entry rounded to bf16)
        att = layer.self_attn
        y = layer.input_layernorm(x)
        shp = (1, 1, -1, s.head_dim)
        q = att.q_proj(y).view(shp).transpose(1, 2)
        k = att.k_proj(y).view(shp).transpose(1, 2)
        v = att.v_proj(y).view(shp).transpose(1, 2)
        q, k = m.apply_rotary_pos_emb(q, k, cos, sin)
        # the library builds its rotary table in float32, so rotated vectors agree to float32 accuracy only
        np.testing.assert_allclose(res["q"], q.reshape(-1).numpy(), atol=5e-6)
        np.testing.assert_allclose(res["k"], k.reshape(-1).numpy(), atol=5e-6)
        np.testing.assert_allclose(res["v"], v.reshape(-1).numpy(), atol=5e-6)  # the library's RMSNorm works in float32
        # the oracle stored the new entry at slot L, rounded by the library's rule
        k_new = torch.from_numpy(res["k"].astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        if orc.real == np.float32:
            np.testing.assert_array_equal(kc[:, L].reshape(-1), k_new)
        Kall, Vall = widen(kc)[None, :, :L + 1], widen(vc)[None, :, :L + 1]
        a, _ = m.eager_attention_forward(att, q, Kall, Vall, None, scaling=s.head_dim ** -0.5, dropout=0.0)
        a = a.reshape(1, 1, -1)
        np.testing.assert_allclose(res["attn"], a.reshape(-1).numpy(), atol=1e-5)
        x1 = x + att.o_proj(a)
        x2 = x1 + layer.mlp(layer.post_attention_layernorm(x1))
        np.testing.assert_allclose(res["x1"], x1.reshape(-1).numpy(), atol=1e-5)
        np.testing.assert_allclose(res["x2"], x2.reshape(-1).numpy(), atol=2e-5)


def test_step_front_and_back_vs_library(orc, tiny):
    """Embedding gather, dual RMSNorm, concatenation order (hidden half first), 2d->d projection, final norm and the
    compressed head, recomputed with torch float64 library ops from the oracle's own decoder-layer output."""
    s, w, act = tiny["shape"], tiny["w"], tiny["act"]
    L = int(act["kv_len"][0])
    kc, vc = act["k_cache"][0].copy(), act["v_cache"][0].copy()
    hb = act["hidden_in"][0]
    token = int(act["token_in"][0])
    res = orc.step(synth.bf16_bits_to_f32(hb).astype(orc.real), token, kc, vc, L, tiny["ids"], trace=True)
    d = s.d_model
    c = torch.cat([F.rms_norm(widen(hb), (d,), widen(w["g_hnorm"]), eps=s.rms_eps),
                   F.rms_norm(widen(w["embed"][token]), (d,), widen(w["g_enorm"]), eps=s.rms_eps)])
    np.testing.assert_allclose(res["c"], c.numpy(), atol=tol(orc, 3e-6, 1e-12))
    np.testing.assert_allclose(res["x"], F.linear(c, widen(w["w_proj"])).numpy(), atol=tol(orc, 5e-6, 1e-12))
    hhat = F.rms_norm(torch.from_numpy(res["x2"].astype(np.float64)), (d,), widen(w["g_final_norm"]), eps=s.rms_eps)
    np.testing.assert_allclose(res["hhat"], hhat.numpy(), atol=tol(orc, 5e-6, 1e-12))
    z = F.linear(hhat, widen(w["lm_head"])[torch.from_numpy(tiny["ids"]).long()]).numpy()
    np.testing.assert_allclose(res["logits"], z, atol=tol(orc, 2e-5, 1e-11))
    assert res["draft"] == int(tiny["ids"][int(np.argmax(res["logits"]))])


def test_step_degenerate_weights(orc, tiny):
    """W_o = W_d = 0 leaves the projection output untouched: hhat = RMSNorm(W_p c; g_f).
    With no prior context the attention output is the new value row as stored (bf16)."""
    s, act = tiny["shape"], tiny["act"]
    w = dict(tiny["w"])
    w["w_o"] = np.zeros_like(w["w_o"])
    w["w_down"] = np.zeros_like(w["w_down"])
    prec = "f32" if orc.real == np.float32 else "f64"
    o = Oracle(s, w, act["kv_capacity"], prec)
    kc, vc = act["k_cache"][0].copy(), act["v_cache"][0].copy()
    h = synth.bf16_bits_to_f32(act["hidden_in"][0]).astype(o.real)
    res = o.step(h, 5, kc, vc, 128, tiny["ids"], trace=True)
    np.testing.assert_array_equal(res["x2"], res["x"])
    np.testing.assert_allclose(res["hhat"], o.rmsnorm(res["x"], w["g_final_norm"]), rtol=0, atol=0)
    kc0, vc0 = np.zeros_like(kc), np.zeros_like(vc)
    res = orc.step(h, 5, kc0, vc0, 0, tiny["ids"], trace=True)
    v_stored = synth.bf16_bits_to_f32(vc0[:, 0])  # [Hkv][hd]
    want = np.repeat(v_stored, s.n_q_heads // s.n_kv_heads, axis=0).reshape(-1)
    np.testing.assert_array_equal(res["attn"], want.astype(orc.real))
    assert np.abs(want - res["v"].reshape(s.n_kv_heads, -1).repeat(2, axis=0).reshape(-1)).max() < 0.01


# ---------------------------------------------------------------- recursion / weight sharing (Sec. 2.1, 2.3)
def test_chain_equals_manual_feedback_of_single_steps(orc, tiny):
    """One K=3 call equals three K=1 calls fed back by hand: same function at every depth, only the position
    and the inputs change; step k>1 takes the previous output hidden state and the previous draft token."""
    s, act, ids = tiny["shape"], tiny["act"], tiny["ids"]
    K = 3
    kc, vc = act["k_cache"].copy(), act["v_cache"].copy()
    full = orc.chain(K, act["hidden_in"], act["token_in"], kc, vc, act["kv_len"], ids)
    kc2, vc2 = act["k_cache"].copy(), act["v_cache"].copy()
    h = synth.bf16_bits_to_f32(act["hidden_in"][0]).astype(orc.real)
    tok = int(act["token_in"][0])
    L = int(act["kv_len"][0])
    for k in range(K):
        r = orc.step(h, tok, kc2[0], vc2[0], L + k, ids)
        assert r["draft"] == full["draft"][0, k]
        np.testing.assert_array_equal(r["logits"], full["logits"][0, k])
        np.testing.assert_array_equal(r["hhat"], full["hidden"][0, k])
        assert r["margin"] == full["margin"][0, k]
        h, tok = r["hhat"], r["draft"]
    np.testing.assert_array_equal(kc, kc2)
    np.testing.assert_array_equal(vc, vc2)
    # cache: exactly K new slots per sequence, everything else untouched
    assert np.array_equal(kc[0, :, :L], act["k_cache"][0, :, :L]) and np.all(kc[0, :, L + K:] == 0)
    assert np.all(kc[0, :, L:L + K].reshape(s.n_kv_heads, -1).any(axis=1))


def test_chain_forced_tokens_and_alt_reading(orc, tiny):
    act, ids = tiny["act"], tiny["ids"]
    K = 3
    base = orc.chain(K, act["hidden_in"], act["token_in"], act["k_cache"].copy(), act["v_cache"].copy(),
                     act["kv_len"], ids)
    # forcing the tokens the chain drafted anyway changes nothing
    same = orc.chain(K, act["hidden_in"], act["token_in"], act["k_cache"].copy(), act["v_cache"].copy(),
                     act["kv_len"], ids, forced=base["draft"][:, :K - 1])
    np.testing.assert_array_equal(base["logits"], same["logits"])
    # forcing other tokens changes steps 2.. but not step 1
    other = (base["draft"][:, :K - 1] + 7) % tiny["shape"].vocab_size
    diff = orc.chain(K, act["hidden_in"], act["token_in"], act["k_cache"].copy(), act["v_cache"].copy(),
                     act["kv_len"], ids, forced=other)
    np.testing.assert_array_equal(base["logits"][:, 0], diff["logits"][:, 0])
    assert np.abs(base["logits"][:, 1] - diff["logits"][:, 1]).max() > 1e-3
    # alternative reading (recurring vector taken before the final norm) is a different function from step 2 on
    prec = "f32" if orc.real == np.float32 else "f64"
    alt = Oracle(tiny["shape"], tiny["w"], act["kv_capacity"], prec, recur_pre_norm=True)
    r = alt.chain(K, act["hidden_in"], act["token_in"], act["k_cache"].copy(), act["v_cache"].copy(),
                  act["kv_len"], ids)
    np.testing.assert_array_equal(base["logits"][:, 0], r["logits"][:, 0])
    assert np.abs(base["logits"][:, 1] - r["logits"][:, 1]).max() > 1e-6


def test_batch_sequences_are_independent(orc, tiny):
    s, ids = tiny["shape"], tiny["ids"]
    wl = tiny["wl"]
    act = synth.make_activations(wl, ctx=np.array([128, 37, 0], dtype=np.int32), capacity=192)
    o = Oracle(s, tiny["w"], 192, "f32" if orc.real == np.float32 else "f64")
    full = o.chain(2, act["hidden_in"], act["token_in"], act["k_cache"].copy(), act["v_cache"].copy(),
                   act["kv_len"], ids)
    for b in range(3):
        one = o.chain(2, act["hidden_in"][b:b + 1], act["token_in"][b:b + 1], act["k_cache"][b:b + 1].copy(),
                      act["v_cache"][b:b + 1].copy(), act["kv_len"][b:b + 1], ids)
        np.testing.assert_array_equal(one["logits"][0], full["logits"][b])


# ---------------------------------------------------------------- first step over several positions
def _extend_inputs(tiny, B, m_max, seed):
    """Position-major synthetic inputs for the multi-position first step: bf16 hiddens like the workload's, tokens."""
    s = tiny["shape"]
    rng = np.random.default_rng(seed)
    hid = rand_bits(rng, (m_max, B, s.d_model), std=float(synth.bf16_bits_to_f32(tiny["act"]["hidden_in"]).std()))
    tok = rng.integers(0, s.vocab_size, size=(m_max, B)).astype(np.int32)
    return hid, tok


def test_extend_one_position_is_the_first_chain_step(orc, tiny):
    act = tiny["act"]
    B = len(act["kv_len"])
    kc1, vc1 = act["k_cache"].copy(), act["v_cache"].copy()
    kc2, vc2 = act["k_cache"].copy(), act["v_cache"].copy()
    ch = orc.chain(1, act["hidden_in"], act["token_in"], kc1, vc1, act["kv_len"], tiny["ids"])
    ex = orc.extend(act["hidden_in"][None], act["token_in"][None], np.ones(B, np.int32), kc2, vc2, act["kv_len"],
                    tiny["ids"])
    np.testing.assert_array_equal(ex["draft"][0], ch["draft"][:, 0])
    np.testing.assert_array_equal(ex["logits"][0], ch["logits"][:, 0])
    np.testing.assert_array_equal(ex["hidden"][0], ch["hidden"][:, 0])
    np.testing.assert_array_equal(kc1, kc2)
    np.testing.assert_array_equal(vc1, vc2)
    np.testing.assert_array_equal(ex["kv_len"], act["kv_len"] + 1)


def test_extend_vs_hf_qwen2_block_forward(orc, tiny):
    """Four new positions through the Hugging Face Qwen2 layer in float64 against the oracle's position-by-position
    result.  (1) One forward over the whole block with a causal mask on top of the prior cache: the library keeps
    the new keys and values unrounded, hence the loose tolerance of the single-position pin.  (2) Position by
    position with the library's own pieces on the cache as the oracle left it (new entries rounded to bf16): tight,
    and a visible range that is one slot short is three orders of magnitude outside it.  Together they pin the
    bookkeeping: position j sits at slot L + j, is rotated for that position, and sees slots 0 .. L + j."""
    from transformers.cache_utils import DynamicCache
    s, w, act = tiny["shape"], tiny["w"], tiny["act"]
    m_lib, cfg, layer, rot = _hf_layer(s, w)
    mm = 4
    L = int(act["kv_len"][0])
    hid, tok = _extend_inputs(tiny, 1, mm, 11)
    kc, vc = act["k_cache"][:1].copy(), act["v_cache"][:1].copy()
    ex = orc.extend(hid, tok, np.array([mm], np.int32), kc, vc, act["kv_len"][:1], tiny["ids"])
    # the decoder layer's input at each position: dual norm + concat + projection (pinned on its own above)
    d = s.d_model
    xs = []
    for j in range(mm):
        c = torch.cat([F.rms_norm(widen(hid[j, 0]), (d,), widen(w["g_hnorm"]), eps=s.rms_eps),
                       F.rms_norm(widen(w["embed"][tok[j, 0]]), (d,), widen(w["g_enorm"]), eps=s.rms_eps)])
        xs.append(F.linear(c, widen(w["w_proj"])))
    x = torch.stack(xs)[None]                                   # [1][m][d]
    pos = torch.arange(L, L + mm)[None]
    cos, sin = rot(x, pos)
    fin = lambda t: F.rms_norm(t.reshape(-1, d), (d,), widen(w["g_final_norm"]), eps=s.rms_eps).numpy()
    with torch.no_grad():
        # (1) the block at once
        cache = DynamicCache(config=cfg)
        cache.update(widen(act["k_cache"])[0:1, :, :L], widen(act["v_cache"])[0:1, :, :L], 0)
        mask = torch.zeros(1, 1, mm, L + mm, dtype=torch.float64)
        for j in range(mm):
            mask[0, 0, j, L + j + 1:] = -math.inf
        out = layer(x, attention_mask=mask, position_ids=pos, past_key_values=cache, use_cache=True,
                    position_embeddings=(cos, sin))
        out = out[0] if isinstance(out, tuple) else out
        hhat = fin(out)
        scale = float(np.abs(hhat).max())
        assert np.abs(ex["hidden"][:, 0] - hhat).max() < 2e-3 * scale
        # (2) position by position on the stored cache
        att = layer.self_attn
        y = layer.input_layernorm(x)
        shp = (1, mm, -1, s.head_dim)
        q = att.q_proj(y).view(shp).transpose(1, 2)
        k = att.k_proj(y).view(shp).transpose(1, 2)
        q, k = m_lib.apply_rotary_pos_emb(q, k, cos, sin)
        if orc.real == np.float32:   # the stored keys are the library's keys for positions L .. L+m-1, rounded
            k_bits = k.float().to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)[0]   # [Hkv][m][hd]
            assert (kc[0][:, L:L + mm] != k_bits).mean() < 0.01     # float32 rotary table: a rare last-bit flip
        for j in range(mm):
            for visible, close in ((L + j + 1, True), (L + j, False)):
                Kall, Vall = widen(kc)[0:1, :, :visible], widen(vc)[0:1, :, :visible]
                a, _ = m_lib.eager_attention_forward(att, q[:, :, j:j + 1], Kall, Vall, None,
                                                     scaling=s.head_dim ** -0.5, dropout=0.0)
                x1 = x[:, j:j + 1] + att.o_proj(a.reshape(1, 1, -1))
                x2 = x1 + layer.mlp(layer.post_attention_layernorm(x1))
                gap = float(np.abs(ex["hidden"][j, 0] - fin(x2)[0]).max())
                assert (gap < 3e-5 * scale) if close else (gap > 3e-4 * scale), (j, visible, gap)


def test_extend_is_causal_splittable_and_ragged(orc, tiny):
    act = tiny["act"]
    B = len(act["kv_len"])
    mm = 5
    hid, tok = _extend_inputs(tiny, B, mm, 12)
    ext = np.array([(3 * b + 5) % (mm + 1) for b in range(B)], np.int32)   # 0 .. mm, ragged
    ext[0] = mm
    if B > 1:
        ext[1] = 0
    kc, vc = act["k_cache"].copy(), act["v_cache"].copy()
    full = orc.extend(hid, tok, ext, kc, vc, act["kv_len"], tiny["ids"])
    assert not full["overflow"]
    np.testing.assert_array_equal(full["kv_len"], act["kv_len"] + ext)
    for b in range(B):
        assert (full["draft"][:ext[b], b] >= 0).all() and (full["draft"][ext[b]:, b] == -1).all()
        # nothing outside the new slots was written
        L = int(act["kv_len"][b])
        np.testing.assert_array_equal(kc[b, :, :L], act["k_cache"][b, :, :L])
        np.testing.assert_array_equal(kc[b, :, L + ext[b]:], act["k_cache"][b, :, L + ext[b]:])
    # two calls (the first two positions, then the rest) leave the same bits behind
    kc2, vc2 = act["k_cache"].copy(), act["v_cache"].copy()
    first = np.minimum(ext, 2)
    a = orc.extend(hid[:2], tok[:2], first, kc2, vc2, act["kv_len"], tiny["ids"])
    b2 = orc.extend(hid[2:], tok[2:], ext - first, kc2, vc2, a["kv_len"], tiny["ids"])
    np.testing.assert_array_equal(kc, kc2)
    np.testing.assert_array_equal(vc, vc2)
    for b in range(B):
        np.testing.assert_array_equal(full["logits"][:first[b], b], a["logits"][:first[b], b])
        np.testing.assert_array_equal(full["logits"][2:ext[b], b], b2["logits"][:ext[b] - first[b], b])
    # later positions do not reach back: new inputs at positions >= 2 leave positions 0, 1 as they were
    hid3, tok3 = hid.copy(), tok.copy()
    hid3[2:], tok3[2:] = _extend_inputs(tiny, B, mm - 2, 13)
    kc3, vc3 = act["k_cache"].copy(), act["v_cache"].copy()
    c = orc.extend(hid3, tok3, ext, kc3, vc3, act["kv_len"], tiny["ids"])
    np.testing.assert_array_equal(c["logits"][:2], full["logits"][:2])
    assert np.abs(c["logits"][2:, 0] - full["logits"][2:, 0]).max() > 0


def test_extend_overflow_leaves_the_sequence_alone(orc, tiny):
    act = tiny["act"]
    cap = act["kv_capacity"]
    B = min(2, len(act["kv_len"]))
    hid, tok = _extend_inputs(tiny, B, 3, 14)
    kv = act["kv_len"][:B].copy()
    kv[0] = cap - 2                                              # three new positions do not fit
    kc, vc = act["k_cache"][:B].copy(), act["v_cache"][:B].copy()
    res = orc.extend(hid, tok, np.full(B, 3, np.int32), kc, vc, kv, tiny["ids"])
    assert res["overflow"] and (res["draft"][:, 0] == -1).all() and res["kv_len"][0] == cap - 2
    np.testing.assert_array_equal(kc[0], act["k_cache"][0])
    if B > 1:
        assert (res["draft"][:, 1] >= 0).all() and res["kv_len"][1] == kv[1] + 3


# ---------------------------------------------------------------- high-frequency list from a token stream
def test_build_subset_brute_force_and_invariants():
    """Counts and the top-n rule against plain Python on small streams (dict counting, sort with an explicit key),
    including ties at the cut, ids that never occur, ids out of range, n = 0 and n = V."""
    rng = np.random.default_rng(5)
    for V, N, n in ((7, 40, 3), (16, 10, 12), (50, 2000, 50), (50, 2000, 0), (33, 500, 5)):
        toks = rng.integers(-2, V + 2, size=N)
        got = orc_mod.build_subset(toks, V, n)
        cnt = {}
        bad = 0
        for t in toks.tolist():
            if 0 <= t < V:
                cnt[t] = cnt.get(t, 0) + 1
            else:
                bad += 1
        ranked = sorted(range(V), key=lambda v: (-cnt.get(v, 0), v))
        assert got["invalid"] == bad
        assert got["counts"].tolist() == [cnt.get(v, 0) for v in range(V)]
        assert got["ids"].tolist() == sorted(ranked[:n])
        # what makes it a top-n list: nothing outside occurs more often than anything inside
        inside = set(got["ids"].tolist())
        if 0 < n < V:
            assert min(cnt.get(v, 0) for v in inside) >= max(cnt.get(v, 0) for v in range(V) if v not in inside)
    # a worked example: counts 3, 1, 3, 0, 2 -> top-3 = ids {0, 2, 4}; top-2 takes the tie 0, 2 (not 4)
    ex = [0, 0, 0, 1, 2, 2, 2, 4, 4]
    assert orc_mod.build_subset(ex, 5, 3)["ids"].tolist() == [0, 2, 4]
    assert orc_mod.build_subset(ex, 5, 2)["ids"].tolist() == [0, 2]
    assert orc_mod.build_subset(ex, 5, 4)["ids"].tolist() == [0, 1, 2, 4]
    assert orc_mod.build_subset(ex, 5, 5)["ids"].tolist() == [0, 1, 2, 3, 4]


def test_token_stream_is_long_tailed_and_list_covers_it():
    """The synthetic corpus has the long tail Sec. 2.2 describes: a fifth of the vocabulary covers most occurrences,
    and the list built from one half of a stream covers the other half almost as well."""
    V, N = 4096, 1 << 18
    s = synth.make_token_stream(V, N, seed=1)
    a, b = s[: N // 2], s[N // 2:]
    lst = orc_mod.build_subset(a, V, V // 5)
    assert lst["invalid"] == 0 and len(set(lst["ids"].tolist())) == V // 5
    assert (np.diff(lst["ids"]) > 0).all()
    cover_a = np.isin(a, lst["ids"]).mean()
    cover_b = np.isin(b, lst["ids"]).mean()
    assert cover_a > 0.75 and cover_b > cover_a - 0.02
    s2 = synth.make_token_stream(V, 1000, seed=2, invalid_every=10)
    assert orc_mod.build_subset(s2, V, 10)["invalid"] == 100


# ---------------------------------------------------------------- teacher-forced K-step forward and its loss
def test_loss_weights_eq2():
    """Eq. (2) with the paper's decay 0.6 and depth 3 (Sec. 3.1): 1 : 0.6 : 0.36 normalised."""
    a = orc_mod.loss_weights(3, 0.6)
    np.testing.assert_allclose(a, np.array([1.0, 0.6, 0.36]) / 1.96, rtol=1e-15)
    assert abs(a.sum() - 1.0) < 1e-15 and abs(a[1] / a[0] - 0.6) < 1e-15
    np.testing.assert_allclose(orc_mod.loss_weights(1, 0.3), [1.0])
    np.testing.assert_allclose(orc_mod.loss_weights(4, 1.0), [0.25] * 4)


def test_train_loss_against_library_cross_entropy_and_hand_fed_steps(orc, tiny):
    """The K-step teacher-forced forward: (1) step 1 is the block-of-positions routine from an empty cache, and its
    loss is torch's cross_entropy of those logits against t_{i+2}; (2) step 2 at every position is a single step
    fed by hand with the step-1 output of the SAME position and t_{i+2}, attending only step-2 keys, scored
    against t_{i+3}; (3) the total is the Eq. (2) mix.  Shifting any label or input token by one breaks (1) or (2)."""
    s, act = tiny["shape"], tiny["act"]
    n, K, beta = 6, 3, 0.6
    rng = np.random.default_rng(21)
    hid = rand_bits(rng, (n, s.d_model), std=float(synth.bf16_bits_to_f32(act["hidden_in"]).std()))
    tok = rng.integers(0, s.vocab_size, size=n + K + 1).astype(np.int32)
    res = orc_mod.train_loss(orc, hid, tok, K, beta)
    cap = act["kv_capacity"]
    zero = lambda: (np.zeros((1, s.n_kv_heads, cap, s.head_dim), np.uint16), np.zeros((1, s.n_kv_heads, cap, s.head_dim), np.uint16))
    # (1)
    kc, vc = zero()
    ex = orc.extend(hid[:, None], tok[1:1 + n, None], np.array([n], np.int32), kc, vc, np.zeros(1, np.int32), None)
    np.testing.assert_array_equal(res["logits"][0], ex["logits"][:, 0])
    ce1 = F.cross_entropy(torch.from_numpy(ex["logits"][:, 0].astype(np.float64)), torch.from_numpy(tok[2:2 + n]).long())
    assert abs(res["ce"][0] - float(ce1)) < 1e-12
    # (2)
    kc2, vc2 = zero()
    for i in range(n):
        r = orc.step(ex["hidden"][i, 0], int(tok[i + 2]), kc2[0], vc2[0], i, None)
        np.testing.assert_array_equal(res["logits"][1][i], r["logits"])
    ce2 = F.cross_entropy(torch.from_numpy(res["logits"][1].astype(np.float64)), torch.from_numpy(tok[3:3 + n]).long())
    assert abs(res["ce"][1] - float(ce2)) < 1e-12
    ce3 = F.cross_entropy(torch.from_numpy(res["logits"][2].astype(np.float64)), torch.from_numpy(tok[4:4 + n]).long())
    # (3)
    want = (1.0 * float(ce1) + 0.6 * float(ce2) + 0.36 * float(ce3)) / 1.96
    assert abs(res["loss"] - want) < 1e-12
    # a label off by one is a different number altogether
    wrong = F.cross_entropy(torch.from_numpy(ex["logits"][:, 0].astype(np.float64)), torch.from_numpy(tok[1:1 + n]).long())
    assert abs(float(wrong) - res["ce"][0]) > 1e-3


def test_train_loss_uniform_head_is_log_vocab(tiny):
    """With every row of the output head equal, all logits of a position are equal and each CE_k is ln |V| exactly,
    whatever the rest of the head computes: the loss is ln |V| for any beta."""
    s = tiny["shape"]
    w = dict(tiny["w"])
    w["lm_head"] = np.tile(tiny["w"]["lm_head"][:1], (s.vocab_size, 1))
    o = Oracle(s, w, tiny["act"]["kv_capacity"], "f64")
    rng = np.random.default_rng(22)
    hid = rand_bits(rng, (4, s.d_model))
    tok = rng.integers(0, s.vocab_size, size=4 + 2 + 1).astype(np.int32)
    res = orc_mod.train_loss(o, hid, tok, 2, 0.6)
    np.testing.assert_allclose(res["ce"], math.log(s.vocab_size), rtol=1e-12)
    assert abs(res["loss"] - math.log(s.vocab_size)) < 1e-10


def test_f32_oracle_within_rounding_of_f64(tiny):
    act, ids = tiny["act"], tiny["ids"]
    outs = {}
    for prec in ("f32", "f64"):
        o = Oracle(tiny["shape"], tiny["w"], act["kv_capacity"], prec)
        outs[prec] = o.chain(3, act["hidden_in"], act["token_in"], act["k_cache"].copy(), act["v_cache"].copy(),
                             act["kv_len"], ids, forced=np.array([[11, 12]]))
    assert np.abs(outs["f32"]["logits"] - outs["f64"]["logits"]).max() < 2e-4


# ---------------------------------------------------------------- shapes (Sec. 3.1)
def test_parameter_counts_match_paper():
    g = golden()
    s = synth.SEVEN_B
    head = synth.head_param_count(s)
    assert round(head / 1e6, 1) == g["mtp_head_params_millions"]
    d, F_, V = s.d_model, s.d_ffn, s.vocab_size
    layer = (s.q_dim * d + 2 * s.kv_dim * d + s.q_dim + 2 * s.kv_dim) + d * s.q_dim + 3 * F_ * d + 2 * d
    total = 36 * layer + d + 2 * V * d + head
    assert round(total / 1e6, 1) == g["total_params_millions"]
    assert head / total < g["trainable_fraction_upper"]
    # without q/k/v biases the printed total would not come out
    no_bias = total - 37 * (s.q_dim + 2 * s.kv_dim)
    assert round(no_bias / 1e6, 1) != g["total_params_millions"]


# ---------------------------------------------------------------- acceptance (Sec. 2.3 verification)
def _accept_definition(dr, tg, L, mode):
    K = len(dr)
    a = 0
    for j in range(K):
        if all(dr[m] == tg[m] for m in range(j + 1)):
            a = j + 1
    out = list(dr[:a]) + [tg[a]] + [-1] * (K - a)
    if mode == 0:
        return a, out, L + min(a + 1, K), int(a == K)
    return a, out, L, 0


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("mode", [0, 1])
def test_accept_exhaustive(K, mode):
    pats = list(itertools.product([0, 1], repeat=K))
    B = len(pats)
    rng = np.random.default_rng(K)
    draft = rng.integers(0, 1000, size=(B, K)).astype(np.int32)
    target = rng.integers(0, 1000, size=(B, K + 1)).astype(np.int32)
    for b, p in enumerate(pats):
        for j in range(K):
            target[b, j] = draft[b, j] if p[j] else draft[b, j] + 1 + j
    L = rng.integers(0, 5000, size=B).astype(np.int32)
    r = orc_mod.accept(draft, target, L, mode)
    for b in range(B):
        a, out, newL, pend = _accept_definition(draft[b].tolist(), target[b].tolist(), int(L[b]), mode)
        assert r["accept_len"][b] == a
        assert r["out_tokens"][b].tolist() == out
        assert r["kv_len"][b] == newL
        assert r["pending"][b] == pend


def test_accept_reproduces_paper_tau():
    """Per-position acceptance 81/56/36 % with sequential acceptance gives tau = 1 + .81 + .56 + .36 = 2.73, the
    mean the paper prints for K=3 with the full vocabulary; matches after the first miss must not count."""
    g = golden()
    p = [g["accept_rate_pos1"], g["accept_rate_pos2"], g["accept_rate_pos3"]]
    counts = {3: round(p[2] * 100), 2: round((p[1] - p[2]) * 100), 1: round((p[0] - p[1]) * 100)}
    counts[0] = 100 - sum(counts.values())
    rows_d, rows_t = [], []
    for a, c in counts.items():
        for _ in range(c):
            dr = [10, 20, 30]
            tg = [10, 20, 30, 40]
            if a < 3:
                tg[a] = 99  # first miss at position a+1; later positions still agree and must be ignored
            rows_d.append(dr)
            rows_t.append(tg)
    r = orc_mod.accept(np.array(rows_d), np.array(rows_t), np.zeros(100, np.int32), 0)
    tau = g["baseline_tau"] + r["accept_len"].mean()
    assert round(float(tau), 2) == g["mean_tau_k3_full_vocab"]


def test_accept_expected_length_closed_form():
    """With independent per-position agreement p, E[a] = sum_j p^j (1.952 for p=0.8, K=3; 1.94117 for p=0.7, K=5)."""
    for name, want in (("c3_7b_b16", 1.952), ("c5_7b_b64", 1.94117)):
        wl = synth.WORKLOADS[name]
        K, p = wl.draft_steps, wl.accept_prob
        assert abs(sum(p ** j for j in range(1, K + 1)) - want) < 1e-5
        B = 40000
        drafts = np.random.default_rng(0).integers(0, wl.shape.vocab_size, size=(B, K))
        tg = synth.make_targets(wl, drafts)
        r = orc_mod.accept(drafts, tg, np.zeros(B, np.int32), 0)
        assert abs(r["accept_len"].mean() - want) < 0.03
