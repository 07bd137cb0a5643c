"""GPU parity at the benchmark's sizes (70B/7B-shape pair), run with -m gpu.

The oracle cannot hold the full-depth pair, so the check is split the way the scope allows:
  * depth-truncated pair of the SAME widths (d 8192, 64 query / 8 KV heads, FFN 28672, vocab 32000; draft d 4096):
    every logit row of the verify forward against the oracle;
  * the full-depth pair in the launch configuration the benchmark times (4096-token prompt, window 7, two streams):
    properties that hold at any size - a multi-token verify equals sequential single-token forwards, rollback then
    re-verify is bit-exact, greedy PEARL = greedy SD = greedy autoregressive decoding, overlapped = serialised,
    and the matrix-core prompt pass leaves the same cache as verify-sized prompt forwards.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import transformer
from tests.util import gpu_available, np_weights as np_weights_of, oracle_model

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]


def _rel_err(got, ref):
    rng = ref.max(axis=-1) - ref.min(axis=-1)
    return float((np.abs(got - ref).max(axis=-1) / rng).max())


@pytest.mark.parametrize("prefill_mode", [1, 0], ids=["dense_prefill", "chunked_prefill"])
@pytest.mark.parametrize("name", ["70b_7b", "33b_1b", "7b_1b", "small"])
def test_full_width_truncated_pair_matches_oracle(name, prefill_mode):
    """Every workload pair at its real widths (depth cut to 2 target layers and 1 draft layer so that the fp32
    oracle can hold it): GQA 64/8 and 32/4, MHA with 56 and 16 heads, head_dim 64 and 128, vocab 32000 and 32256.
    The prompt goes in through the matrix-core path or as 32-token verify forwards; either way every later logit
    row must match the oracle."""
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    cfg = synth.config(name, depth=2, draft_depth=1)
    print(f"full-width truncated pair {name}: generating weights on the GPU", flush=True)
    tw, dw = synth.make_pair(cfg, device="cuda")            # bf16, the values both sides get
    target, draft = harness.build_pair(cfg, weights=(tw, dw))
    cpu = lambda w: {"tok_embed": w["tok_embed"].cpu(), "lm_head": w["lm_head"].cpu(), "final_norm": w["final_norm"].cpu(),
                     "layers": [{k: v.cpu() for k, v in lay.items()} for lay in w["layers"]]}
    tm = oracle_model(cpu(tw), cfg.target)
    dm = oracle_model(cpu(dw), cfg.draft)
    del tw, dw
    cfg.n_prompt, cfg.n_generate = 150, 64
    ctx = harness.make_context(cfg, target, draft, 8)
    ctx.set_option(amd.SPEC_OPT_PREFILL, prefill_mode)
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 7).tolist()
    extra = synth.prompt_tokens(16, cfg.target.vocab, 8).tolist()
    ctx.prefill(prompt)
    print("oracle prefill", flush=True)
    oc = transformer.CachedModel(tm, 256)
    oc.feed(prompt[:-1])
    worst = 0.0
    pos = 0
    for m in (1, 7, 8):                                     # pre-verify, post-verify at gamma 7, SD at gamma 7
        toks = ([prompt[-1]] + extra)[pos:pos + m]
        pos += m
        got = ctx.verify(toks, want_logits=True)
        ref = oc.feed(toks)
        worst = max(worst, _rel_err(got, ref))
        print(f"  M={m}: logit error / range so far {worst:.2e}", flush=True)
    assert worst <= 2e-2
    # the draft model: its first sampled token against the oracle's distribution
    od = transformer.CachedModel(dm, 256)
    od.feed(prompt[:-1])
    from oracle import sampling
    q = sampling.probs(od.feed([prompt[-1]])[0], 1.0, 1.0)
    ctx.rewind(len(prompt))
    x = ctx.draft_step(0.37, want_token=True)
    if sampling.sample_margin(q, 0.37) > 1e-3:
        assert x == sampling.sample(q, 0.37)
    ctx.close()


def _cpu_weights(w):
    return {"tok_embed": w["tok_embed"].cpu(), "lm_head": w["lm_head"].cpu(), "final_norm": w["final_norm"].cpu(),
            "layers": [{k: v.cpu() for k, v in lay.items()} for lay in w["layers"]]}


@pytest.mark.parametrize("name,self_draft", [("70b_7b", False), ("70b_7b", True), ("33b_1b", False)],
                         ids=["70b_7b", "70b_first_layer_as_draft", "33b_1b"])
def test_full_width_truncated_pair_decodes_like_the_oracle(name, self_draft):
    """PEARL and SD (gamma 4, temperature 1, the pair's own accept / reject decisions) on the real widths and the real
    vocabulary, depth cut to 2 target layers so that the fp32 oracle can hold the pair: every forward of the run
    against the oracle forward (2e-2 of the row's range), every committed token against the oracle's loop on the
    library's logits - draws over 32000 ids, acceptance ratios and residual resampling on model-produced rows.
    With an independent random-init draft the acceptance rate is what chance gives; with the target's own first layer
    as the draft model (shared embedding and LM head) it lies in the range trained pairs show."""
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    from tests.test_gpu_loops import lockstep_run
    from tests.util import EXACT_MARGIN
    cfg = synth.config(name, depth=2, draft_depth=1)
    if self_draft:
        cfg.draft_from_target_layers = 1
        cfg.draft = synth._truncate(cfg.target, 1)
    tw, dw = synth.make_pair(cfg, device="cuda")
    target, draft = harness.build_pair(cfg, weights=(tw, dw))
    tm = oracle_model(_cpu_weights(tw), cfg.target)
    dm = oracle_model(_cpu_weights(dw), cfg.draft)
    del tw, dw
    cfg.n_prompt, cfg.n_generate = 100, 64
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 9).tolist()
    for algo in (amd.ALGO_PEARL, amd.ALGO_SD):
        print(f"{name} self_draft={self_draft} algo={algo}", flush=True)
        agreed, splits, wt, wd, modes = lockstep_run(amd, harness, cfg, target, draft, tm, dm, algo, 4, 1.0,
                                                     n_total=40, seed=31, prompt=prompt, first_segment=40)
        print(f"  {agreed} steps identical, {splits} splits within {EXACT_MARGIN} of a flip; worst logit error "
              f"target {wt:.2e} draft {wd:.2e}; modes {sorted(map(str, modes))}", flush=True)
        assert splits <= 2 and agreed >= 8 * max(1, splits)
        if self_draft and algo == amd.ALGO_PEARL:
            assert modes >= {"pre-verify", "post-verify"}


@pytest.fixture(scope="module")
def small_pair_full_depth():
    """The small pair at its full depth (24 target layers of width 2048, draft = its first 4 layers, vocab 32000),
    the oracle in fp32 (5.4 GB), and the oracle's caches after the 512-token prompt."""
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    cfg = synth.config("small")
    print("small pair at full depth: weights", flush=True)
    tw, dw = synth.make_pair(cfg, device="cuda")
    target, draft = harness.build_pair(cfg, weights=(tw, dw))
    tm = oracle_model(_cpu_weights(tw), cfg.target)
    dm = oracle_model(_cpu_weights(dw), cfg.draft)
    del tw, dw
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    print("small pair at full depth: oracle prompt pass (511 tokens, 24 + 4 layers)", flush=True)
    caches = []
    for m in (tm, dm):
        c = transformer.CachedModel(m, cfg.n_prompt + 160)
        c.feed(prompt[:-1])
        caches.append(c)
    return amd, harness, cfg, target, draft, tm, dm, prompt, caches


def _copy_cache(c):
    """A second oracle cache with the same contents (the weights are shared, not copied)."""
    n = transformer.CachedModel(c.model, c.cache.k.shape[1])
    n.cache.k[:, :c.len] = c.cache.k[:, :c.len]
    n.cache.v[:, :c.len] = c.cache.v[:, :c.len]
    n.cache.len = c.len
    return n


@pytest.mark.parametrize("prefill_mode", [1, 0], ids=["dense_prefill", "chunked_prefill"])
def test_small_pair_at_full_depth_verify_rows_match_the_oracle(small_pair_full_depth, prefill_mode):
    """24 layers deep, behind the 512-token prompt (either prompt path): verify forwards of 1, 5 and 9 rows."""
    amd, harness, cfg, target, draft, tm, dm, prompt, _ = small_pair_full_depth
    ctx = harness.make_context(cfg, target, draft, 8, extra_seq=64)
    ctx.set_option(amd.SPEC_OPT_PREFILL, prefill_mode)
    ctx.prefill(prompt)
    oc = _copy_cache(small_pair_full_depth[8][0])
    extra = synth.prompt_tokens(16, cfg.target.vocab, 8).tolist()
    worst, pos = 0.0, 0
    for m in (1, 5, 9):
        toks = ([prompt[-1]] + extra)[pos:pos + m]
        pos += m
        got = ctx.verify(toks, want_logits=True)
        ref = oc.feed(toks)
        worst = max(worst, _rel_err(got, ref))
        print(f"  24 layers, M={m}: logit error / range so far {worst:.2e}", flush=True)
    ctx.close()
    assert worst <= 2e-2


# (algo, gamma, temperature, prompt path): the workload's own settings (greedy and temperature 1, windows 4 and 8), and
# temperature 0.3, where the distributions are as peaked as a trained model's
SMALL_FULL_DEPTH_CASES = [(1, 4, 0.3, 1), (2, 4, 0.3, 1), (2, 4, 0.3, 0), (2, 8, 0.0, 1), (1, 8, 0.0, 0), (1, 4, 1.0, 1),
                          (2, 8, 1.0, 1)]


@pytest.mark.parametrize("algo,gamma,temperature,prefill_mode", SMALL_FULL_DEPTH_CASES)
def test_small_pair_at_full_depth_decodes_like_the_oracle(small_pair_full_depth, algo, gamma, temperature, prefill_mode):
    """SD / PEARL with the pair's own decisions at the full 24-layer depth behind the 512-token prompt: every target
    forward (1, gamma and gamma + 1 rows) and every draft forward against the fp32 oracle, every committed token
    against the oracle's loop on the library's logits.  At temperature 1 this random-init pair spreads its mass
    almost evenly over the 32000 ids: CDF edges lie 3e-5 apart, every draw sits within 2e-5 of one, and the last
    bits of exp() already move a few per cent of the draws to a neighbouring id - there the test can only demand
    that each split is such a close call; greedy runs must agree token for token, and at temperature 0.3 splits must
    be rare."""
    from tests.test_gpu_loops import lockstep_run
    from tests.util import EXACT_MARGIN
    amd, harness, cfg, target, draft, tm, dm, prompt, filled = small_pair_full_depth
    caches = (_copy_cache(filled[0]), _copy_cache(filled[1]))
    n_total = 40 if temperature == 1.0 else 96
    agreed, splits, wt, wd, modes = lockstep_run(amd, harness, cfg, target, draft, tm, dm, algo, gamma, temperature,
                                                 n_total=n_total, seed=cfg.seed_uniform, prompt=prompt,
                                                 prefill_mode=prefill_mode, first_segment=n_total, oracle_caches=caches)
    print(f"algo={algo} gamma={gamma} T={temperature} prefill={prefill_mode}: {agreed} steps identical, {splits} splits "
          f"within {EXACT_MARGIN} of a flip; worst logit error target {wt:.2e} draft {wd:.2e}", flush=True)
    if temperature == 0.0:
        assert splits == 0 and agreed >= 10
    elif temperature < 1.0:
        assert splits <= 1 and agreed >= 24
    else:
        assert agreed >= 12


@pytest.mark.parametrize("gamma,k,temperature", [(4, 3, 0.6), (8, 5, 1.0)])
def test_small_pair_at_full_depth_pre_verifies_several_drafts_like_the_oracle(small_pair_full_depth, gamma, k, temperature):
    """PEARL with pre-verify over guessed continuations (closing remark of Section 4.3) on the full 24-layer pair, the
    pair's own decisions (at temperatures 0.6 and 1 it accepts often enough for pre-verify steps to take several drafts), guesses from
    the caller (the step's drafts, one in three corrupted), in lockstep with the oracle's reading of it."""
    from tests.test_gpu_loops import lockstep_run
    from tests.test_gpu_multi_preverify import scripted_hooks
    from tests.util import EXACT_MARGIN
    amd, harness, cfg, target, draft, tm, dm, prompt, filled = small_pair_full_depth
    caches = (_copy_cache(filled[0]), _copy_cache(filled[1]))
    gpu, oracle, seen = scripted_hooks(k, cfg.target.vocab)
    agreed, splits, wt, wd, modes = lockstep_run(amd, harness, cfg, target, draft, tm, dm, amd.ALGO_PEARL_GUESS, gamma,
                                                 temperature, n_total=96, seed=cfg.seed_uniform + 3, prompt=prompt,
                                                 prefill_mode=1, first_segment=96, oracle_caches=caches,
                                                 oracle_loop=oracle, gpu_steps=gpu, gpu_first=True)
    acc_pre = sorted({s["n_accepted"] for s in seen if s["mode"] == amd.SPEC_MODE_PRE})
    rows_post = sorted({s["rows"] for s in seen if s["mode"] == amd.SPEC_MODE_POST})
    print(f"gamma={gamma} k={k} T={temperature}: {agreed} steps identical, {splits} splits within {EXACT_MARGIN} of a "
          f"flip; pre-verify acceptances seen {acc_pre}, post-verify rows seen {rows_post}; worst logit error target "
          f"{wt:.2e} draft {wd:.2e}", flush=True)
    assert agreed >= 10 and (temperature == 1.0 or splits <= 1)     # (temperature 1: see the test above)
    assert max(acc_pre) >= 2 and len(rows_post) >= 2


DEPTH_TOL_FP32 = {2: 2e-2, 4: 2e-2, 8: 4e-2}    # against the fp32 oracle: the stated 2e-2 holds up to 4 layers at these widths
DEPTH_TOL_BF16 = 2e-2                              # against the oracle with bf16 activations, any depth measured


def test_logit_error_against_the_oracle_as_depth_grows_at_70b_widths():
    """The 70B-shape target at 2, 4 and 8 layers (the deeper models share the shallower ones' layers) against the
    oracle: verify forwards of 1 and 7 rows behind a 150-token prompt.  Three distances per depth: library vs fp32
    oracle, library vs the oracle with bf16 activations (the same rounding points as a bf16 deployment), and the two
    oracles against each other.  In a random-init network a perturbation grows from layer to layer, so bf16
    activations alone (oracle vs oracle, no library involved) leave the 2e-2 of the fp32 logits' range behind at
    about 8 layers of these widths; the library must stay as close to the fp32 oracle as the bf16-activation oracle
    does (within a factor), and closer to that oracle than to the fp32 one."""
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    cfg = synth.config("70b_7b", depth=8, draft_depth=1)
    print("70B widths, 8 layers: generating weights on the GPU", flush=True)
    tw, dw = synth.make_pair(cfg, device="cuda")
    target8, draft = harness.build_pair(cfg, weights=(tw, dw))
    w8 = np_weights_of(_cpu_weights(tw))
    del tw, dw
    cfg.n_prompt, cfg.n_generate = 150, 32
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 7).tolist()
    extra = synth.prompt_tokens(8, cfg.target.vocab, 8).tolist()
    curve = {}
    for depth in (2, 4, 8):
        shape = synth._truncate(cfg.target, depth)
        tgt = target8.prefix(depth, shape)
        cfg_k = synth.config("70b_7b", depth=depth, draft_depth=1)
        cfg_k.n_prompt, cfg_k.n_generate = cfg.n_prompt, cfg.n_generate
        ctx = harness.make_context(cfg_k, tgt, draft, 8)
        ctx.set_option(amd.SPEC_OPT_PREFILL, 0)      # the prompt through the same kernels as the verify forwards
        ctx.prefill(prompt)
        wk = dict(w8, layers=w8["layers"][:depth])
        mk = lambda r: transformer.CachedModel(transformer.Model(wk, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                                                                 shape.rope_theta, shape.rms_eps, act_bf16=r), 256)
        o32, o16 = mk(False), mk(True)
        print(f"  depth {depth}: oracle prompt passes", flush=True)
        o32.feed(prompt[:-1])
        o16.feed(prompt[:-1])
        e32 = e16 = eoo = 0.0
        for toks in ([prompt[-1]], extra[:7]):
            got = ctx.verify(toks, want_logits=True)
            r32, r16 = o32.feed(toks), o16.feed(toks)
            e32, e16, eoo = max(e32, _rel_err(got, r32)), max(e16, _rel_err(got, r16)), max(eoo, _rel_err(r16, r32))
        ctx.close()
        curve[depth] = (e32, e16, eoo)
        print(f"  depth {depth}: library vs fp32 oracle {e32:.2e}, library vs bf16-activation oracle {e16:.2e}, "
              f"bf16-activation oracle vs fp32 oracle {eoo:.2e} (max |dlogit| / row range)", flush=True)
    print(f"depth curve at 70B widths: {curve}", flush=True)
    for depth, (e32, e16, eoo) in curve.items():
        assert e32 <= DEPTH_TOL_FP32[depth], (depth, e32)
        assert e32 <= 1.5 * eoo + 2e-3, (depth, e32, eoo)     # no further from fp32 than bf16 activations put anyone
        assert e16 <= DEPTH_TOL_BF16 and e16 <= 0.75 * e32 + 1e-3, (depth, e16, e32)   # measured: about half of e32


@pytest.fixture(scope="module")
def full_depth_pair():
    """The benchmark's pair at its full depth (80 + 32 layers, 151 GB of bf16 weights on the GPU)."""
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    cfg = synth.config("70b_7b")
    print("full-depth pair: building 151 GB of weights", flush=True)
    target, draft = harness.build_pair(cfg)
    return amd, harness, cfg, target, draft


def _np_layer(shape, seed, l, stage):
    """Layer l of the generator's weights as fp32 NumPy arrays (the bf16 values, upcast): made on the GPU by the same
    counter-based generator that filled the library's model, one layer at a time.  `stage`: dict of pinned host
    tensors, one per matrix, reused from layer to layer (a pageable copy of 3.4 GB per layer is what this test
    would otherwise spend most of its time on); the arrays returned are views of them, valid until the next call."""
    import torch
    lay = {}

    def cv(name, t):
        if name not in stage:
            stage[name] = torch.empty(t.shape, dtype=torch.float32, pin_memory=True)
        stage[name].copy_(t.float())
        return stage[name].numpy()

    for name in ("attn_norm", "ffn_norm"):
        lay[name] = cv(name, synth.gain_tensor(shape.d_model, seed, 16 * l + synth._SLOT[name], torch.bfloat16, "cuda"))
    for name, shp in synth.layer_matrix_shapes(shape).items():
        lay[name] = cv(name, synth.normal_tensor(shp, 0.02, seed, 16 * l + synth._SLOT[name], torch.bfloat16, "cuda"))
    return lay


def _streamed_oracle_logits(shape, seed, seq):
    """Logits [len(seq), vocab] of one causal pass over `seq` from the plain fp32 oracle and from the oracle with
    bf16 activations, the layers generated, used by both and dropped one at a time."""
    import torch
    cv = lambda t: np.ascontiguousarray(t.float().cpu().numpy())
    gen = lambda name: synth.normal_tensor((shape.vocab, shape.d_model), 0.02, seed, synth._GLOBAL[name],
                                           torch.bfloat16, "cuda")
    glob = {"tok_embed": cv(gen("tok_embed")), "lm_head": cv(gen("lm_head")),
            "final_norm": cv(synth.gain_tensor(shape.d_model, seed, synth._GLOBAL["final_norm"], torch.bfloat16, "cuda")),
            "layers": []}
    models, caches, hs = [], [], []
    for act_bf16 in (False, True):
        m = transformer.Model(glob, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.rope_theta, shape.rms_eps,
                              act_bf16=act_bf16)
        m.layers = [None] * shape.n_layers          # the cache is sized from this; the layers arrive one by one
        models.append(m)
        caches.append(transformer.KVCache(m, len(seq)))
        hs.append(m.tok_embed[np.asarray(seq, dtype=np.int64)])
    stage = {}
    for l in range(shape.n_layers):
        w = _np_layer(shape, seed, l, stage)
        for i, m in enumerate(models):
            hs[i] = transformer.layer_forward(m, caches[i], l, w, hs[i], 0)
        del w
        if l % 8 == 7:
            d = float(np.abs(hs[1] - hs[0]).max() / np.abs(hs[0]).max())
            print(f"  oracle layer {l + 1}/{shape.n_layers}: residual streams of the two oracles differ by {d:.2e} of "
                  f"the largest entry", flush=True)
    return transformer.head(models[0], hs[0]), transformer.head(models[1], hs[1])


@pytest.mark.parametrize("which", ["target", "draft"])
def test_full_depth_models_against_the_oracle_layer_by_layer(full_depth_pair, which):
    """The 80-layer 70B-shape target itself (and the 32-layer 7B-shape draft model) against the oracle.  The fp32
    oracle cannot hold 70e9 weights at once, but it can take them one layer at a time: the test generates layer l
    again (same generator, same seeds), runs oracle.transformer.layer_forward for the plain fp32 oracle and for the
    oracle with bf16 activations, and drops the layer.  One causal pass over the whole sequence (96 prompt tokens, the
    frontier, 7 more tokens) gives the oracle's logits of the rows the library then computes as a one-token and a
    seven-token forward - after either prompt path.  In a random-init network of these widths bf16 activation
    rounding grows with depth (the two oracles part by eoo, no library involved); the library must be no further
    from the fp32 oracle than that, within a factor - a mistake in any layer (a wrong gain vector, a misplaced head,
    a stale cache row) gives errors of the order of the logit range itself."""
    amd, harness, cfg, target, draft = full_depth_pair
    shape, seed, model = (cfg.target, cfg.seed_target, target) if which == "target" else (cfg.draft, cfg.seed_draft, draft)
    prompt = synth.prompt_tokens(97, shape.vocab, 41).tolist()      # 96 cached positions: two K/V pages, three chunks
    extra = synth.prompt_tokens(7, shape.vocab, 42).tolist()
    r32, r16 = _streamed_oracle_logits(shape, seed, prompt + extra)
    rows = slice(len(prompt) - 1, len(prompt) + len(extra))     # the frontier's row and the seven after it
    eoo = _rel_err(r16[rows], r32[rows])
    # the model in question sits in the context's target slot: spec_verify returns its logits
    cfg_m = synth.PairConfig(cfg.name, shape, cfg.draft, n_prompt=128, n_generate=32, gamma=7)
    ctx = harness.make_context(cfg_m, model, draft, 8, temperature=0.0)
    for mode, label in ((0, "chunked prompt pass"), (1, "dense prompt pass")):
        ctx.set_option(amd.SPEC_OPT_PREFILL, mode)
        ctx.prefill(prompt)
        got = np.concatenate([ctx.verify([prompt[-1]], want_logits=True), ctx.verify(extra, want_logits=True)])
        e32, e16 = _rel_err(got, r32[rows]), _rel_err(got, r16[rows])
        agree = int((got.argmax(-1) == r32[rows].argmax(-1)).sum())
        print(f"  {which}, {shape.n_layers} layers, {label}: library vs fp32 oracle {e32:.2e}, library vs "
              f"bf16-activation oracle {e16:.2e}, bf16-activation oracle vs fp32 oracle {eoo:.2e} (max |dlogit| / row "
              f"range); arg-max equal to the fp32 oracle's in {agree} of 8 rows", flush=True)
        assert e32 <= 1.5 * eoo + 2e-3, (label, e32, eoo)
        assert e16 <= 1.5 * eoo + 2e-3, (label, e16, eoo)
    ctx.close()


def test_full_depth_pair_properties_in_benchmark_configuration(full_depth_pair):
    amd, harness, cfg, target, draft = full_depth_pair
    gamma = 7
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    toks = synth.prompt_tokens(gamma, cfg.target.vocab, 3).tolist()
    ctx = harness.make_context(cfg, target, draft, 16, temperature=0.0, extra_seq=64)
    print("prefill 4096 tokens", flush=True)
    ctx.prefill(prompt)
    n0 = len(prompt)
    base = ctx.kv_len(amd.SPEC_TARGET)
    # (1) multi-token verify == sequential single-token forwards
    multi = ctx.verify(toks, want_logits=True)
    ctx.rollback_kv(amd.SPEC_TARGET, base)
    seq = np.concatenate([ctx.verify([t], want_logits=True) for t in toks])
    err = _rel_err(multi, seq)
    print(f"  multi-token vs sequential: {err:.2e} of the logit range", flush=True)
    # Two bf16 evaluation orders of an 80-layer random-init network: the attention split differs between M = 7 and
    # M = 1, the tiny fp32 differences pass bf16 rounding points differently and grow roughly like sqrt(depth)
    # (2 layers of the same widths sit at 6e-3 .. 9e-3 against the fp32 oracle).  Bound: a few times that growth.
    assert err < 6e-2
    # (2) rollback then re-verify is bit-exact, pages come back
    free0 = ctx.free_pages(amd.SPEC_TARGET)
    ctx.verify(list(range(1, 33)))
    ctx.rollback_kv(amd.SPEC_TARGET, base)
    again = ctx.verify(toks, want_logits=True)
    assert np.array_equal(multi, again)
    ctx.rewind(n0)
    assert ctx.free_pages(amd.SPEC_TARGET) >= free0
    # (3) greedy: PEARL == SD == AR, token for token (Section 3.2: lossless), two streams
    n_gen = 12
    uni = synth.make_uniforms(n_gen + 1, gamma, cfg.seed_uniform)
    outs = {}
    for algo in (amd.ALGO_AR, amd.ALGO_SD, amd.ALGO_PEARL):
        ctx.rewind(n0)
        outs[algo], st = ctx.generate(algo, gamma, n_gen, uni)
        print(f"  algo {algo}: {st['steps']:.0f} steps", flush=True)
    # The three loops evaluate the same arg-max through different batch shapes (1, gamma + 1 and gamma rows); at 80
    # layers those bf16 evaluation orders differ by up to a few 1e-2 of the logit range (see (1)), so the sequences
    # may part at a near-tie of the target's top two logits - and only there.
    for other in (amd.ALGO_SD, amd.ALGO_PEARL):
        a, b = outs[amd.ALGO_AR], outs[other]
        i = next((k for k in range(n_gen) if a[k] != b[k]), None)
        if i is None:
            continue
        ctx.rewind(n0)
        row = ctx.verify([prompt[-1]] + a[:i], want_logits=True)[-1]
        gap = abs(float(row[a[i]]) - float(row[b[i]])) / float(row.max() - row.min())
        print(f"  algo {other} parts from AR at token {i}: logit gap {gap:.2e} of the range", flush=True)
        # both choices sit within the evaluation-order noise of the row's maximum (they need not be its top two:
        # a third logit can lie between them)
        top_gap = (float(row.max()) - min(float(row[a[i]]), float(row[b[i]]))) / float(row.max() - row.min())
        assert gap < 6e-2 and top_gap < 6e-2
    # (3b) the two prompt paths fill equivalent caches: `multi` came after the matrix-core prompt pass (the default
    # for this shape); the same verify after 128 verify-sized prompt forwards is another bf16 evaluation order
    ctx.set_option(amd.SPEC_OPT_PREFILL, 0)
    ctx.prefill(prompt)
    chunked = ctx.verify(toks, want_logits=True)
    err = _rel_err(multi, chunked)
    print(f"  dense vs chunked prompt pass: {err:.2e} of the logit range", flush=True)
    # Here every one of the 4095 cached K / V rows differs in rounding between the two runs, not only the new
    # tokens' rows as in (1).  Bound: two independent bf16 evaluation orders, each sqrt(80 / 2) times the 6e-3 ..
    # 8e-3 that 2 layers of these widths show against the fp64 oracle, i.e. sqrt(2) * 6.3 * 8e-3 = 7e-2 for a
    # typical logit, and this is the maximum over 7 x 32000 of them (observed 3.4e-2 and 7.7e-2 with two
    # different, equally accurate, orders of the RMSNorm arithmetic).
    assert err < 1.5e-1
    ctx.close()
    # (4) sampled PEARL: overlapped streams == one stream, bit for bit
    res = []
    for serial in (True, False):
        c2 = harness.make_context(cfg, target, draft, 16, serial=serial, extra_seq=64)
        c2.prefill(prompt)
        out, st = c2.generate(amd.ALGO_PEARL, gamma, n_gen, uni)
        res.append(out)
        c2.close()
    assert res[0] == res[1]
