"""Pins for the oracle's transformer forward (CPU only).

Each check compares the oracle with something other than itself: an independently written
full-sequence (cache-free, masked) forward in torch float64 with complex-number RoPE, closed
forms, and algebraic invariants.
"""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import transformer
from tests.util import np_weights, oracle_model


def _tiny_shape(n_layers=2, d=64, hq=4, hkv=2, f=96, v=50):
    return synth.ModelShape(n_layers, d, hq, hkv, f, v)


def _weights(shape, seed=5, std=0.2):
    w = synth.make_weights(shape, seed, torch.float32, std=std)
    # non-trivial norm gains so that a dropped gain would show
    g = torch.Generator().manual_seed(seed)
    for lay in w["layers"]:
        lay["attn_norm"] = 1.0 + 0.3 * torch.randn(shape.d_model, generator=g)
        lay["ffn_norm"] = 1.0 + 0.3 * torch.randn(shape.d_model, generator=g)
    w["final_norm"] = 1.0 + 0.3 * torch.randn(shape.d_model, generator=g)
    return w


def brute_force_logits(w, shape, tokens):
    """Textbook decoder over the whole sequence at once: no cache, explicit causal mask,
    RoPE as multiplication of complex pairs (x_i + i x_{i+D/2}) by exp(i * pos * theta^(-2i/D))."""
    T = len(tokens)
    f64 = lambda t: t.to(torch.float64)
    H, Hkv, D = shape.n_heads, shape.n_kv_heads, shape.head_dim
    h = f64(w["tok_embed"])[torch.tensor(tokens, dtype=torch.long)]
    pos = torch.arange(T, dtype=torch.float64)
    freq = shape.rope_theta ** (-2.0 * torch.arange(D // 2, dtype=torch.float64) / D)
    rot = torch.polar(torch.ones(T, D // 2, dtype=torch.float64), pos[:, None] * freq[None, :])   # [T, D/2]

    def norm(x, g):
        return x * torch.rsqrt((x ** 2).mean(-1, keepdim=True) + shape.rms_eps) * f64(g)

    def rotate(x):      # x [T, heads, D]
        z = torch.complex(x[..., :D // 2], x[..., D // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    for lay in w["layers"]:
        a = norm(h, lay["attn_norm"])
        q = rotate(torch.einsum("td,od->to", a, f64(lay["wq"])).view(T, H, D))
        k = rotate(torch.einsum("td,od->to", a, f64(lay["wk"])).view(T, Hkv, D))
        v = torch.einsum("td,od->to", a, f64(lay["wv"])).view(T, Hkv, D)
        k = k.repeat_interleave(H // Hkv, dim=1)       # query head j uses kv head j // group
        v = v.repeat_interleave(H // Hkv, dim=1)
        s = torch.einsum("thd,shd->hts", q, k) / math.sqrt(D)
        s = s.masked_fill(~mask[None], float("-inf"))
        o = torch.einsum("hts,shd->thd", torch.softmax(s, dim=-1), v).reshape(T, H * D)
        h = h + torch.einsum("tk,dk->td", o, f64(lay["wo"]))
        b = norm(h, lay["ffn_norm"])
        g = torch.einsum("td,fd->tf", b, f64(lay["w_gate"]))
        u = torch.einsum("td,fd->tf", b, f64(lay["w_up"]))
        h = h + torch.einsum("tf,df->td", torch.nn.functional.silu(g) * u, f64(lay["w_down"]))
    return torch.einsum("td,vd->tv", norm(h, w["final_norm"]), f64(w["lm_head"])).numpy()


@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 2), (4, 1)])
def test_forward_matches_independent_full_sequence_model(hq, hkv):
    shape = _tiny_shape(hq=hq, hkv=hkv)
    w = _weights(shape)
    toks = synth.prompt_tokens(11, shape.vocab, 3).tolist()
    ref = brute_force_logits(w, shape, toks)
    m = oracle_model(w, shape, dtype=np.float64)
    cm = transformer.CachedModel(m, 32)
    got = np.concatenate([cm.feed(toks[:4]), cm.feed(toks[4:5]), cm.feed(toks[5:])])   # mixed chunking
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-10)


def test_multi_token_verify_equals_sequential_single_token_forwards():
    shape = _tiny_shape()
    w = _weights(shape)
    toks = synth.prompt_tokens(13, shape.vocab, 9).tolist()
    for dtype, tol in ((np.float64, 1e-11), (np.float32, 1e-5)):
        m = oracle_model(w, shape, dtype=dtype)
        a = transformer.CachedModel(m, 32)
        b = transformer.CachedModel(m, 32)
        a.feed(toks[:8]); b.feed(toks[:8])
        multi = a.feed(toks[8:])                                     # gamma+1 = 5 tokens at once
        seq = np.concatenate([b.feed([t]) for t in toks[8:]])
        scale = np.abs(seq).max()
        assert np.abs(multi - seq).max() <= tol * scale
        np.testing.assert_allclose(a.cache.k[:, :13], b.cache.k[:, :13], rtol=0, atol=tol * 10)


def test_rollback_then_refeed_reproduces_logits_and_cache():
    shape = _tiny_shape()
    m = oracle_model(_weights(shape), shape, dtype=np.float64)
    toks = synth.prompt_tokens(12, shape.vocab, 1).tolist()
    a = transformer.CachedModel(m, 32)
    a.feed(toks[:6])
    first = a.feed(toks[6:10])
    a.feed([1, 2, 3])                       # speculate past the point
    a.rollback(6)
    again = a.feed(toks[6:10])              # same shapes => bit-identical
    assert np.array_equal(first, again)
    with pytest.raises(ValueError):
        a.rollback(11)


def test_rope_preserves_norm_and_depends_on_relative_position_only():
    rng = np.random.default_rng(0)
    D = 16
    q = rng.standard_normal((1, 1, D))
    k = rng.standard_normal((1, 1, D))
    for theta in (10000.0, 500.0):
        base = None
        for m_pos, n_pos in ((7, 3), (11, 7), (104, 100)):
            qr = transformer.rope(q, [m_pos], theta)
            kr = transformer.rope(k, [n_pos], theta)
            assert abs(np.linalg.norm(qr) - np.linalg.norm(q)) < 1e-12
            dot = float((qr * kr).sum())
            base = dot if base is None else base
            assert abs(dot - base) < 1e-10
    # position 0 is the identity; pair (i, i + D/2) rotates by pos * theta^(-2i/D)
    assert np.array_equal(transformer.rope(q, [0], 10000.0), q)
    e = np.zeros((1, 1, D)); e[0, 0, 1] = 1.0
    r = transformer.rope(e, [5], 10000.0)
    ang = 5 * 10000.0 ** (-2.0 / D)
    assert abs(r[0, 0, 1] - math.cos(ang)) < 1e-12 and abs(r[0, 0, 1 + D // 2] - math.sin(ang)) < 1e-12


def test_norm_and_activation_closed_forms():
    x = np.full((1, 8), 3.0)
    np.testing.assert_allclose(transformer.rmsnorm(x, np.arange(8.0), 0.0), np.arange(8.0)[None], rtol=1e-15)
    x = np.array([[3.0, -4.0]])
    np.testing.assert_allclose(transformer.rmsnorm(x, np.ones(2), 1e-5), x / math.sqrt(12.5 + 1e-5), rtol=1e-15)
    assert transformer.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(transformer.silu(np.array([1.0, -2.0])),
                               [1 / (1 + math.exp(-1)), -2 / (1 + math.exp(2))], rtol=1e-15)


def test_attention_with_zero_queries_averages_values():
    """With W_q = 0 every score is 0, so each head outputs the mean of the visible values."""
    shape = _tiny_shape(n_layers=1, hq=2, hkv=1)
    w = _weights(shape)
    w["layers"][0]["wq"] = torch.zeros_like(w["layers"][0]["wq"])
    m = oracle_model(w, shape, dtype=np.float64)
    toks = [3, 9, 27, 4]
    cm = transformer.CachedModel(m, 8)
    got = cm.feed(toks)
    # recompute by hand from the cached values
    wl = m.layers[0]
    h = m.tok_embed[toks]
    vmean = np.cumsum(cm.cache.v[0, :4, 0], axis=0) / np.arange(1, 5)[:, None]          # [T, D]
    o = np.concatenate([vmean, vmean], axis=-1)                                        # both query heads
    h = h + o @ wl["wo"].T
    b = transformer.rmsnorm(h, wl["ffn_norm"], m.rms_eps)
    h = h + (transformer.silu(b @ wl["w_gate"].T) * (b @ wl["w_up"].T)) @ wl["w_down"].T
    ref = transformer.rmsnorm(h, m.final_norm, m.rms_eps) @ m.lm_head.T
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    shape_g = _tiny_shape(hq=4, hkv=2)
    w = _weights(shape_g)
    shape_m = _tiny_shape(hq=4, hkv=4)
    wm = {"tok_embed": w["tok_embed"], "lm_head": w["lm_head"], "final_norm": w["final_norm"], "layers": []}
    D = shape_g.head_dim
    for lay in w["layers"]:
        l2 = dict(lay)
        for name in ("wk", "wv"):
            l2[name] = lay[name].view(2, D, -1).repeat_interleave(2, dim=0).reshape(4 * D, -1)
        wm["layers"].append(l2)
    toks = synth.prompt_tokens(7, shape_g.vocab, 2).tolist()
    a = transformer.CachedModel(oracle_model(w, shape_g, np.float64), 8).feed(toks)
    b = transformer.CachedModel(oracle_model(wm, shape_m, np.float64), 8).feed(toks)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-12)


def test_byte_model_of_the_benchmark_against_the_papers_kv_cache_example():
    """The byte counts behind every GB/s figure of the benchmark.  KV cache: the paper's appendix on
    resource-constrained scenarios works out 2 x 2 x 32 x 1 x 8 x 1024 x 128 bytes (K and V, 2-byte elements, 32
    layers, batch 1, 8 KV heads, 1024 tokens, head_dim 128), about 0.13 GB, for an 8B GQA model; weights: every
    matrix of a layer once plus the LM head, 2 bytes each."""
    import bench
    llama8b = synth.ModelShape(32, 4096, 32, 8, 14336, 128256)
    assert llama8b.head_dim == 128
    kv = 1024 * llama8b.kv_bytes_per_token()
    assert kv == 2 * 2 * 32 * 1 * 8 * 1024 * 128 and abs(kv / 1e9 - 0.13) < 0.005
    # the 70B shape of the benchmark: 4096 B per token and layer, 80 layers
    t70 = synth.config("70b_7b").target
    assert t70.kv_bytes_per_token() == 80 * 4096 == 327680
    per_layer = 8192 * (64 + 2 * 8) * 128 + 64 * 128 * 8192 + 3 * 8192 * 28672
    assert t70.params_per_layer() == per_layer and t70.streamed_params() == 80 * per_layer + 32000 * 8192
    n, m = 4096, 7
    assert bench.forward_bytes(t70, n, m) == 2 * t70.streamed_params() + (n + m) * 327680 + m * 32000 * 4


def test_bf16_round_is_round_to_nearest_even_on_the_upper_16_bits():
    f = lambda v: float(transformer.bf16_round(np.array([v], dtype=np.float32))[0])
    assert f(1.0) == 1.0 and f(-2.5) == -2.5 and f(0.0) == 0.0
    ulp = 2.0 ** -7                                    # spacing of bfloat16 in [1, 2): 8 significant bits
    assert f(1.0 + 0.49 * ulp) == 1.0 and f(1.0 + 0.51 * ulp) == 1.0 + ulp
    assert f(1.0 + 0.5 * ulp) == 1.0                   # tie -> even mantissa
    assert f(1.0 + 1.5 * ulp) == 1.0 + 2 * ulp         # tie -> even mantissa (upwards)
    assert f(-(1.0 + 1.5 * ulp)) == -(1.0 + 2 * ulp)
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    r = transformer.bf16_round(x)
    assert np.array_equal(transformer.bf16_round(r), r)                      # idempotent
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)                    # half an ulp, relative
    assert np.array_equal(r, torch.from_numpy(x).to(torch.bfloat16).float().numpy())   # the library conversion
    assert transformer.bf16_round(x.astype(np.float64)).dtype == np.float64


def test_bf16_activation_variant_is_the_same_forward_up_to_rounding_noise():
    """act_bf16 only rounds activations: with it off nothing changes; with it on the logits move by an amount of
    the order of bf16's 2^-9 relative step (not zero, not large), and a multi-token feed still equals token-by-token
    feeds up to that noise."""
    cfg = synth.config("tiny")
    tw, _ = synth.make_pair(cfg)
    w = {"tok_embed": tw["tok_embed"].numpy(), "lm_head": tw["lm_head"].numpy(), "final_norm": tw["final_norm"].numpy(),
         "layers": [{k: v.numpy() for k, v in lay.items()} for lay in tw["layers"]]}
    s = cfg.target
    plain = transformer.Model(w, s.n_heads, s.n_kv_heads, s.head_dim, dtype=np.float64)
    rounded = transformer.Model(w, s.n_heads, s.n_kv_heads, s.head_dim, dtype=np.float64, act_bf16=True)
    toks = synth.prompt_tokens(24, s.vocab, 3).tolist()
    a = transformer.CachedModel(plain, 32).feed(toks)
    b = transformer.CachedModel(rounded, 32).feed(toks)
    rng = a.max(axis=-1) - a.min(axis=-1)
    err = (np.abs(a - b).max(axis=-1) / rng).max()
    assert 2e-4 < err < 8e-3, err
    c = transformer.CachedModel(rounded, 32)
    seq = np.concatenate([c.feed([t]) for t in toks])
    assert (np.abs(seq - b).max(axis=-1) / rng).max() < 8e-3


def test_bf16_activation_noise_grows_with_depth_only_where_the_weights_amplify():
    """What bf16 activations cost against exact arithmetic in a random-init decoder, by depth (no GPU involved).
    With N(0, std^2) matrices a projection multiplies the scale of its (normalised) input by about std * sqrt(d).
    Below 1 (std 0.02 at d = 512) every layer's rounding noise stays what it was: the logit error is flat in depth.
    At 1.81 (std 0.08 at d = 512; the value the benchmark's 70B shape has with std 0.02 at d = 8192) a perturbation
    grows from layer to layer: 1e-2 of the logits' range at 2 layers, past 2e-2 by 8, past 5e-2 by 32.  So a bound
    of 2e-2 against fp32 cannot hold at depth for any bf16-activation implementation of that shape; the GPU tests
    assert it where it can hold and compare deeper stacks with the bf16-activation variant as well."""
    shape = synth.ModelShape(32, 512, 8, 2, 1376, 2048)
    prompt = synth.prompt_tokens(64, shape.vocab, 7).tolist()
    curves = {}
    for std in (0.02, 0.08):
        w = synth.make_weights(shape, 1234, torch.bfloat16, std=std)
        wn = {"tok_embed": w["tok_embed"].float().numpy(), "lm_head": w["lm_head"].float().numpy(),
              "final_norm": w["final_norm"].float().numpy(),
              "layers": [{k: v.float().numpy() for k, v in lay.items()} for lay in w["layers"]]}
        for depth in (2, 8, 32):
            wk = dict(wn, layers=wn["layers"][:depth])
            mk = lambda r, dt: transformer.CachedModel(transformer.Model(wk, 8, 2, 64, dtype=dt, act_bf16=r), 80)
            exact = mk(False, np.float64).feed(prompt)[-8:]
            noisy = mk(True, np.float32).feed(prompt)[-8:]
            rng = exact.max(-1) - exact.min(-1)
            curves[(std, depth)] = float((np.abs(exact - noisy).max(-1) / rng).mean())
    print(curves)
    flat = [curves[(0.02, d)] for d in (2, 8, 32)]
    steep = [curves[(0.08, d)] for d in (2, 8, 32)]
    assert max(flat) < 5e-3 and max(flat) < 1.6 * min(flat)
    assert steep[0] < 1.5e-2 and steep[1] > 1.5 * steep[0] and steep[2] > 1.5 * steep[1] and steep[2] > 3e-2
