"""Pins of the CPU oracle (no GPU): library routines, closed forms, invariants, brute force.

The paper prints no worked numeric example for a stage forward, so none of
these values is the paper's; every pin is a library routine (Hugging Face's
Llama decoder, torch's attention / rms_norm / silu), a closed form, an
invariant the paper's method rests on (Sec. IV-A.2: sub-sequence by
sub-sequence equals the whole prompt at once) or brute force.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from oracle import bruteforce
from paper_2504_08242_amd import synth_inputs as si

SMALL = dict(n_layers=2, d_model=32, n_heads=2, head_dim=16, d_ffn=40, rms_eps=1e-5, rope_theta=1e4)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def run_chunked(cfg, layers, hidden, chunks, max_positions=None):
    st = oracle.OracleStage(cfg, layers, max_positions or hidden.shape[0])
    outs, p = [], 0
    for n in chunks:
        outs.append(st.prefill_chunk(hidden[p:p + n], p))
        p += n
    assert p == hidden.shape[0]
    return np.concatenate(outs, axis=0), st


def compositions(S):
    for cuts in itertools.product([0, 1], repeat=S - 1):
        sizes, run = [], 1
        for c in cuts:
            if c:
                sizes.append(run)
                run = 1
            else:
                run += 1
        sizes.append(run)
        yield sizes


# ----------------------------------------------------------------------------------------------
# Library pin: Hugging Face Llama decoder layers with a DynamicCache (fp64, eager attention).
# ----------------------------------------------------------------------------------------------
def hf_model(cfg, layers):
    from transformers import LlamaConfig
    from transformers.models.llama.modeling_llama import LlamaModel

    hc = LlamaConfig(hidden_size=cfg["d_model"], intermediate_size=cfg["d_ffn"], num_hidden_layers=cfg["n_layers"],
                     num_attention_heads=cfg["n_heads"], num_key_value_heads=cfg["n_heads"],
                     head_dim=cfg["head_dim"], rms_norm_eps=cfg["rms_eps"], rope_theta=cfg["rope_theta"],
                     vocab_size=8, max_position_embeddings=4096, attention_bias=False, mlp_bias=False)
    hc._attn_implementation = "eager"
    m = LlamaModel(hc).double().eval()
    m.norm = torch.nn.Identity()
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj", "w_down": "mlp.down_proj",
             "g_attn": "input_layernorm", "g_mlp": "post_attention_layernorm"}
    with torch.no_grad():
        for li, w in enumerate(layers):
            for ours, theirs in names.items():
                mod = m.layers[li].get_submodule(theirs)
                mod.weight.copy_(torch.from_numpy(np.asarray(w[ours], dtype=np.float64)))
    return m


def hf_cache_kv(cache, layer):
    if hasattr(cache, "layers"):
        return cache.layers[layer].keys[0], cache.layers[layer].values[0]
    return cache.key_cache[layer][0], cache.value_cache[layer][0]


@pytest.mark.parametrize("chunks", [[12], [5, 4, 3], [1, 1, 10]])
def test_oracle_matches_hf_llama_chunked(chunks):
    cfg = dict(SMALL, n_layers=3)
    layers = si.make_layers(cfg, seed=3, weight_std=0.15)
    hidden = si.make_hidden(cfg, seed=3, n_tokens=sum(chunks))
    out, st = run_chunked(cfg, layers, hidden, chunks)

    m = hf_model(cfg, layers)
    from transformers import DynamicCache
    cache = DynamicCache()
    ref, p = [], 0
    with torch.no_grad():
        for n in chunks:
            x = torch.from_numpy(hidden[p:p + n].astype(np.float64))[None]
            r = m(inputs_embeds=x, past_key_values=cache, use_cache=True)
            cache = r.past_key_values
            ref.append(r.last_hidden_state[0].numpy())
            p += n
    ref = np.concatenate(ref, axis=0)
    assert rel_l2(out, ref) < 2e-6
    assert np.max(np.abs(out - ref)) < 2e-5
    for l in range(cfg["n_layers"]):
        k, v = hf_cache_kv(cache, l)
        assert rel_l2(st.kv[l, 0], k.numpy()) < 2e-6
        assert rel_l2(st.kv[l, 1], v.numpy()) < 2e-6


def test_bruteforce_matches_hf_llama():
    cfg = dict(SMALL, n_layers=2)
    layers = si.make_layers(cfg, seed=4, weight_std=0.15)
    hidden = si.make_hidden(cfg, seed=4, n_tokens=9)
    out, k, v = bruteforce.stage_full(cfg, layers, hidden)
    m = hf_model(cfg, layers)
    with torch.no_grad():
        r = m(inputs_embeds=torch.from_numpy(hidden.astype(np.float64))[None], use_cache=True)
    # the library evaluates its rotary cos/sin tables in fp32, hence 1e-6 and not 1e-12
    assert rel_l2(out, r.last_hidden_state[0].numpy()) < 1e-6
    for l in range(cfg["n_layers"]):
        kk, vv = hf_cache_kv(r.past_key_values, l)
        assert rel_l2(k[l], kk.numpy()) < 1e-6
        assert rel_l2(v[l], vv.numpy()) < 1e-6


# ----------------------------------------------------------------------------------------------
# Library pins of single steps.
# ----------------------------------------------------------------------------------------------
def test_attention_definition_matches_torch_sdpa():
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal((3, 11, 16)) for _ in range(3))
    ours = bruteforce.causal_attention(q, k, v)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], is_causal=True)[0].numpy()
    assert np.max(np.abs(ours - ref)) < 1e-12


def test_rmsnorm_matches_torch_and_closed_form():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 48)).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(48)).astype(np.float32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x.astype(np.float64)), (48,),
                                       torch.from_numpy(g.astype(np.float64)), eps=1e-5).numpy()
    assert np.max(np.abs(oracle.rmsnorm(x, g, 1e-5) - ref)) < 1e-6
    assert np.max(np.abs(bruteforce.rmsnorm(x, g, 1e-5) - ref)) < 1e-13
    # constant row c  ->  g * c / sqrt(c^2 + eps)
    c = np.float32(0.37)
    y = oracle.rmsnorm(np.full((1, 48), c, np.float32), g, 1e-5)
    assert np.max(np.abs(y[0] - g * c / np.sqrt(np.float64(c) ** 2 + 1e-5))) < 1e-6
    # unit gain: output rows have RMS 1 up to eps
    y1 = oracle.rmsnorm(x, np.ones(48, np.float32), 1e-5)
    assert np.allclose(np.sqrt(np.mean(y1.astype(np.float64) ** 2, axis=1)), 1.0, atol=1e-4)


def test_silu_matches_torch():
    z = np.linspace(-9, 9, 37)
    assert np.max(np.abs(bruteforce.silu(z) - torch.nn.functional.silu(torch.from_numpy(z)).numpy())) < 1e-14
    assert bruteforce.silu(np.float64(0.0)) == 0.0


def test_linear_matches_numpy_fp64():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 300)).astype(np.float32)
    w = rng.standard_normal((13, 300)).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.max(np.abs(oracle.linear_nt(x, w) - ref)) < 1e-5
    # a transposed operand or a swapped index cannot hide behind symmetry
    assert oracle.linear_nt(x, w).shape == (7, 13)


# ----------------------------------------------------------------------------------------------
# RoPE: closed forms and the relative-position invariant.
# ----------------------------------------------------------------------------------------------
def test_rope_closed_forms():
    rng = np.random.default_rng(5)
    dh = 16
    v = rng.standard_normal((6, dh)).astype(np.float32)
    # position 0 is the identity
    assert np.array_equal(oracle.rope(v, np.zeros(6, np.int64), 1e4), v)
    # each (i, i+dh/2) pair is rotated: as complex numbers, multiplied by exp(i * pos * theta^(-2i/dh))
    pos = np.array([1, 2, 3, 50, 700, 4095])
    got = oracle.rope(v, pos, 1e4).astype(np.float64)
    z = v[:, :dh // 2].astype(np.float64) + 1j * v[:, dh // 2:].astype(np.float64)
    w = z * np.exp(1j * pos[:, None] * (1e4 ** (-np.arange(dh // 2) / (dh / 2)))[None, :])
    assert np.max(np.abs(got[:, :dh // 2] - w.real)) < 1e-6
    assert np.max(np.abs(got[:, dh // 2:] - w.imag)) < 1e-6
    # the first pair turns by exactly `pos` radians, the last by pos * theta^(-(dh-2)/dh)
    e0 = np.zeros((1, dh), np.float32)
    e0[0, 0] = 1.0
    r = oracle.rope(e0, np.array([3]), 1e4)
    assert abs(r[0, 0] - np.cos(3.0)) < 1e-7 and abs(r[0, dh // 2] - np.sin(3.0)) < 1e-7
    e7 = np.zeros((1, dh), np.float32)
    e7[0, dh // 2 - 1] = 1.0
    r = oracle.rope(e7, np.array([1000]), 1e4)
    ang = 1000.0 * 1e4 ** (-(dh - 2) / dh)
    assert abs(r[0, dh // 2 - 1] - np.cos(ang)) < 1e-7 and abs(r[0, dh - 1] - np.sin(ang)) < 1e-7
    # the bruteforce definition agrees
    assert np.max(np.abs(bruteforce.rope(v, pos, 1e4) - got)) < 1e-6


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(6)
    dh = 32
    q = rng.standard_normal((1, dh)).astype(np.float32)
    k = rng.standard_normal((1, dh)).astype(np.float32)

    def score(m, n):
        return float(np.sum(oracle.rope(q, [m], 1e4).astype(np.float64) * oracle.rope(k, [n], 1e4).astype(np.float64)))

    base = score(9, 4)
    for shift in (1, 17, 300):
        assert abs(score(9 + shift, 4 + shift) - base) < 2e-5
    assert abs(score(9, 5) - base) > 1e-3  # and does depend on the distance


# ----------------------------------------------------------------------------------------------
# Brute force: every composition of a short prompt, random compositions of the tiny config.
# ----------------------------------------------------------------------------------------------
def test_every_composition_of_a_short_prompt_equals_the_plain_definition():
    cfg = SMALL
    S = 7
    layers = si.make_layers(cfg, seed=11, weight_std=0.18)  # 1/sqrt(d): scores of std ~1, peaky softmax
    hidden = si.make_hidden(cfg, seed=11, n_tokens=S)
    ref, rk, rv = bruteforce.stage_full(cfg, layers, hidden)
    for chunks in compositions(S):
        out, st = run_chunked(cfg, layers, hidden, chunks)
        assert rel_l2(out, ref) < 2e-6, chunks
        assert rel_l2(st.kv[:, 0], rk) < 2e-6, chunks
        assert rel_l2(st.kv[:, 1], rv) < 2e-6, chunks


def test_tiny_config_four_chunks_equals_one_shot_and_plain_definition():
    cfg = si.TINY
    layers = si.make_layers(cfg, seed=0)
    hidden = si.make_hidden(cfg, seed=0, n_tokens=128)
    ref, rk, rv = bruteforce.stage_full(cfg, layers, hidden)
    one, st1 = run_chunked(cfg, layers, hidden, [128])
    four, st4 = run_chunked(cfg, layers, hidden, [32, 32, 32, 32])
    assert rel_l2(one, ref) < 1e-6 and rel_l2(four, ref) < 1e-6
    assert np.max(np.abs(one - four)) < 1e-5
    assert rel_l2(st1.kv[:, 0], rk) < 1e-6 and rel_l2(st4.kv[:, 1], rv) < 1e-6
    assert np.max(np.abs(st1.kv - st4.kv)) < 1e-5
    rng = np.random.default_rng(0)
    for _ in range(3):
        cuts = np.sort(rng.choice(np.arange(1, 128), size=int(rng.integers(1, 9)), replace=False))
        chunks = np.diff(np.concatenate([[0], cuts, [128]])).tolist()
        out, _ = run_chunked(cfg, layers, hidden, chunks)
        assert rel_l2(out, ref) < 1e-6, chunks


def test_peaky_softmax_variant_of_tiny_config():
    cfg = dict(si.TINY, n_layers=1)
    layers = si.make_layers(cfg, seed=1, weight_std=1.0 / 16.0)  # 1/sqrt(256)
    hidden = si.make_hidden(cfg, seed=1, n_tokens=48)
    ref, _, _ = bruteforce.stage_full(cfg, layers, hidden)
    out, _ = run_chunked(cfg, layers, hidden, [16, 7, 25])
    assert rel_l2(out, ref) < 1e-6


# ----------------------------------------------------------------------------------------------
# Closed forms through the whole stage routine.
# ----------------------------------------------------------------------------------------------
def _single_layer(cfg, seed, **overrides):
    cfg = dict(cfg, n_layers=1)
    layers = si.make_layers(cfg, seed=seed, weight_std=0.2)
    for k, v in overrides.items():
        layers[0][k] = v(layers[0][k]) if callable(v) else v
    return cfg, layers


def test_zero_query_weights_give_running_mean_of_values():
    d = SMALL["d_model"]
    cfg, layers = _single_layer(SMALL, 21, wq=np.zeros((d, d), np.float32), wo=np.eye(d, dtype=np.float32),
                                w_down=np.zeros((d, SMALL["d_ffn"]), np.float32))
    hidden = si.make_hidden(cfg, seed=21, n_tokens=10)
    out, st = run_chunked(cfg, layers, hidden, [4, 6])
    o = out - hidden  # wo = I, w_down = 0  ->  out = x + o
    v = st.kv[0, 1].transpose(1, 0, 2).reshape(10, d).astype(np.float64)  # [S, H*dh]
    running_mean = np.cumsum(v, axis=0) / np.arange(1, 11)[:, None]
    assert np.max(np.abs(o - running_mean)) < 1e-6
    # and V itself is rmsnorm(x) wv^T
    vref = bruteforce.rmsnorm(hidden, layers[0]["g_attn"], cfg["rms_eps"]) @ layers[0]["wv"].astype(np.float64).T
    assert np.max(np.abs(v - vref)) < 1e-6


def test_single_token_attends_to_itself_only():
    d = SMALL["d_model"]
    cfg, layers = _single_layer(SMALL, 22, wo=np.eye(d, dtype=np.float32),
                                w_down=np.zeros((d, SMALL["d_ffn"]), np.float32))
    hidden = si.make_hidden(cfg, seed=22, n_tokens=1)
    out, st = run_chunked(cfg, layers, hidden, [1])
    assert np.max(np.abs((out - hidden)[0] - st.kv[0, 1, :, 0, :].reshape(d))) < 5e-7  # fp32 rounding of x + o


def test_identical_tokens_give_identical_attention_rows():
    d = SMALL["d_model"]
    cfg, layers = _single_layer(SMALL, 23, wo=np.eye(d, dtype=np.float32),
                                w_down=np.zeros((d, SMALL["d_ffn"]), np.float32))
    row = si.make_hidden(cfg, seed=23, n_tokens=1)
    hidden = np.repeat(row, 9, axis=0)
    out, st = run_chunked(cfg, layers, hidden, [3, 3, 3])
    v0 = st.kv[0, 1, :, 0, :].reshape(d)
    assert np.max(np.abs((out - hidden) - v0[None, :])) < 1e-6  # all value rows equal -> softmax weights irrelevant


def test_huge_scores_give_one_hot_softmax_without_overflow():
    d = SMALL["d_model"]
    cfg, layers = _single_layer(SMALL, 24, g_attn=lambda g: g * np.float32(60.0), wo=np.eye(d, dtype=np.float32),
                                w_down=np.zeros((d, SMALL["d_ffn"]), np.float32))
    hidden = si.make_hidden(cfg, seed=24, n_tokens=8)
    out, st = run_chunked(cfg, layers, hidden, [8])
    assert np.all(np.isfinite(out))
    H, dh = cfg["n_heads"], cfg["head_dim"]
    xn = bruteforce.rmsnorm(hidden, layers[0]["g_attn"], cfg["rms_eps"])
    q = bruteforce.rope((xn @ layers[0]["wq"].astype(np.float64).T).reshape(8, H, dh).transpose(1, 0, 2),
                        np.arange(8), 1e4)
    k = st.kv[0, 0].astype(np.float64)
    v = st.kv[0, 1].astype(np.float64)
    o = (out - hidden).reshape(8, H, dh)
    checked = 0
    for h in range(H):
        for t in range(8):
            s = q[h, t] @ k[h, :t + 1].T / np.sqrt(dh)
            top = np.sort(s)[::-1]
            if t == 0 or top[0] - top[1] > 40.0:  # softmax weight of the runner-up below e^-40
                assert np.max(np.abs(o[t, h] - v[h, int(np.argmax(s))])) < 1e-4
                checked += 1
    assert checked >= 4


def test_zero_output_projections_pass_the_input_through_exactly():
    d, f = SMALL["d_model"], SMALL["d_ffn"]
    layers = si.make_layers(SMALL, seed=25)
    for w in layers:
        w["wo"] = np.zeros((d, d), np.float32)
        w["w_down"] = np.zeros((d, f), np.float32)
    hidden = si.make_hidden(SMALL, seed=25, n_tokens=6)
    out, _ = run_chunked(SMALL, layers, hidden, [2, 4])
    assert np.array_equal(out, hidden)


def test_two_stages_chained_equal_one_stage_with_all_layers():
    cfg = dict(SMALL, n_layers=4)
    layers = si.make_layers(cfg, seed=26, weight_std=0.15)
    hidden = si.make_hidden(cfg, seed=26, n_tokens=9)
    whole, _ = run_chunked(cfg, layers, hidden, [4, 5])
    a, _ = run_chunked(dict(cfg, n_layers=1), layers[:1], hidden, [4, 5])
    b, _ = run_chunked(dict(cfg, n_layers=3), layers[1:], a, [9])
    assert np.max(np.abs(whole - b)) < 1e-5


def test_kv_slots_written_are_exactly_the_chunk_positions():
    cfg = SMALL
    layers = si.make_layers(cfg, seed=27)
    hidden = si.make_hidden(cfg, seed=27, n_tokens=5)
    st = oracle.OracleStage(cfg, layers, max_positions=9)
    sentinel = np.float32(-777.25)
    st.kv[...] = sentinel
    st.prefill_chunk(hidden[:2], 0)
    assert np.all(st.kv[:, :, :, 2:, :] == sentinel) and not np.any(st.kv[:, :, :, :2, :] == sentinel)
    before = st.kv.copy()
    st.prefill_chunk(hidden[2:], 2)
    assert np.array_equal(st.kv[:, :, :, :2, :], before[:, :, :, :2, :])
    assert np.all(st.kv[:, :, :, 5:, :] == sentinel) and not np.any(st.kv[:, :, :, 2:5, :] == sentinel)
    with pytest.raises(RuntimeError):
        st.prefill_chunk(hidden, 5)  # 5 + 5 > 9


def test_input_generator_is_seeded_and_bf16_rounding_is_nearest_even():
    a = si.make_weight(si.TINY, 0, 1, "wk")
    b = si.make_weight(si.TINY, 0, 1, "wk")
    assert np.array_equal(a, b) and abs(float(a.std()) - 0.02) < 1e-3
    g = si.make_weight(si.TINY, 0, 0, "g_mlp")
    assert abs(float(g.mean()) - 1.0) < 0.01
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-39, 65504.0], dtype=np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(si.round_to_bf16(x), want)
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(si.round_to_bf16(r), torch.from_numpy(r).to(torch.bfloat16).float().numpy())
    assert np.array_equal(si.bf16_bits_to_f32(si.bf16_bits(si.round_to_bf16(r))), si.round_to_bf16(r))


# ----------------------------------------------------------------------------------------------
# Token tree of a speculative step (Sec. V-A): candidates verified in one forward pass.
# ----------------------------------------------------------------------------------------------
def tree_depths_and_ancestors(parents):
    n = len(parents)
    depth = [0] * n
    anc = [[] for _ in range(n)]
    for t in range(n):
        if parents[t] >= 0:
            depth[t] = depth[parents[t]] + 1
            anc[t] = anc[parents[t]] + [int(parents[t])]
    return depth, anc


def test_tree_oracle_matches_hf_llama_with_ancestor_mask_and_depth_positions():
    """Independent pin: the library decoder, driven with an explicit 4-D mask (prefix + ancestors + self) and
    position ids prefix + depth, on a cache that already holds the prefix."""
    cfg = dict(SMALL, n_layers=3)
    layers = si.make_layers(cfg, seed=11, weight_std=0.15)
    p, n = 7, 13
    parents = si.make_token_tree(n, seed=11)
    hidden = si.make_hidden(cfg, seed=11, n_tokens=p + n)
    st = oracle.OracleStage(cfg, layers, p + n)
    st.prefill_chunk(hidden[:p])
    out = st.prefill_tree(hidden[p:], parents)

    depth, anc = tree_depths_and_ancestors(parents)
    m = hf_model(cfg, layers)
    from transformers import DynamicCache
    cache = DynamicCache()
    with torch.no_grad():
        r = m(inputs_embeds=torch.from_numpy(hidden[:p].astype(np.float64))[None], past_key_values=cache,
              use_cache=True)
        cache = r.past_key_values
        mask = torch.full((1, 1, n, p + n), float("-inf"), dtype=torch.float64)
        mask[..., :p] = 0.0
        for t in range(n):
            for a in anc[t] + [t]:
                mask[0, 0, t, p + a] = 0.0
        pos = torch.tensor([[p + dpt for dpt in depth]])
        r = m(inputs_embeds=torch.from_numpy(hidden[p:].astype(np.float64))[None], attention_mask=mask,
              position_ids=pos, cache_position=torch.arange(p, p + n), past_key_values=cache, use_cache=True)
    ref = r.last_hidden_state[0].numpy()
    assert rel_l2(out, ref) < 2e-6
    assert np.max(np.abs(out - ref)) < 2e-5
    for l in range(cfg["n_layers"]):
        k, v = hf_cache_kv(r.past_key_values, l)
        assert rel_l2(st.kv[l, 0], k.numpy()) < 2e-6   # slot p + t holds node t, K rotated at p + depth(t)
        assert rel_l2(st.kv[l, 1], v.numpy()) < 2e-6


def test_tree_node_equals_last_row_of_the_ordinary_call_on_its_path():
    """What verification relies on: a candidate's output is what the model gives after the tokens on its path."""
    cfg = dict(SMALL, n_layers=2)
    layers = si.make_layers(cfg, seed=12, weight_std=0.15)
    p, n = 5, 16
    parents = si.make_token_tree(n, seed=12)
    hidden = si.make_hidden(cfg, seed=12, n_tokens=p + n)
    st = oracle.OracleStage(cfg, layers, p + n)
    st.prefill_chunk(hidden[:p])
    out = st.prefill_tree(hidden[p:], parents)
    _, anc = tree_depths_and_ancestors(parents)
    assert max(len(a) for a in anc) >= 2 and len(set(parents.tolist())) > 3   # a real tree, not a chain or a star
    for t in range(n):
        path = anc[t] + [t]
        chain = oracle.OracleStage(cfg, layers, p + len(path))
        chain.prefill_chunk(hidden[:p])
        ref = chain.prefill_chunk(hidden[p:][path])
        np.testing.assert_array_equal(out[t], ref[-1])   # same keys in the same order: the same roundings
        for j, a in enumerate(path):                      # and the same cache entries, slot p+a vs position p+j
            np.testing.assert_array_equal(st.kv[:, :, :, p + a], chain.kv[:, :, :, p + j])


def test_chain_shaped_tree_is_the_ordinary_sub_sequence():
    cfg = dict(SMALL, n_layers=2)
    layers = si.make_layers(cfg, seed=13, weight_std=0.15)
    hidden = si.make_hidden(cfg, seed=13, n_tokens=14)
    a = oracle.OracleStage(cfg, layers, 14)
    b = oracle.OracleStage(cfg, layers, 14)
    a.prefill_chunk(hidden[:4]); b.prefill_chunk(hidden[:4])
    oa = a.prefill_chunk(hidden[4:])
    ob = b.prefill_tree(hidden[4:], np.arange(-1, 9))
    np.testing.assert_array_equal(oa, ob)
    np.testing.assert_array_equal(a.kv, b.kv)


def test_siblings_do_not_see_each_other():
    """A star (every candidate follows the prefix directly) is n independent one-token calls at the same position."""
    cfg = dict(SMALL, n_layers=2)
    layers = si.make_layers(cfg, seed=14, weight_std=0.15)
    p, n = 6, 5
    hidden = si.make_hidden(cfg, seed=14, n_tokens=p + n)
    st = oracle.OracleStage(cfg, layers, p + n)
    st.prefill_chunk(hidden[:p])
    out = st.prefill_tree(hidden[p:], [-1] * n)
    for t in range(n):
        one = oracle.OracleStage(cfg, layers, p + 1)
        one.prefill_chunk(hidden[:p])
        np.testing.assert_array_equal(out[t], one.prefill_chunk(hidden[p + t:p + t + 1])[0])


def test_keep_leaves_the_cache_of_the_accepted_path():
    """Sec. V-A step 5: after the rejected candidates are removed the cache is that of the accepted tokens alone."""
    cfg = dict(SMALL, n_layers=2)
    layers = si.make_layers(cfg, seed=15, weight_std=0.15)
    p, n = 5, 16
    parents = si.make_token_tree(n, seed=15)
    hidden = si.make_hidden(cfg, seed=15, n_tokens=p + n + 3)
    _, anc = tree_depths_and_ancestors(parents)
    leaf = max(range(n), key=lambda t: len(anc[t]))
    path = anc[leaf] + [leaf]
    st = oracle.OracleStage(cfg, layers, p + n + 3)
    st.prefill_chunk(hidden[:p])
    st.prefill_tree(hidden[p:p + n], parents)
    st.keep(p, path)
    assert st.kv_len == p + len(path)
    nxt = st.prefill_chunk(hidden[p + n:])
    ref = oracle.OracleStage(cfg, layers, p + n + 3)
    ref.prefill_chunk(hidden[:p])
    ref.prefill_chunk(hidden[p:p + n][path])
    np.testing.assert_array_equal(nxt, ref.prefill_chunk(hidden[p + n:]))
    np.testing.assert_array_equal(st.kv[:, :, :, :st.kv_len], ref.kv[:, :, :, :ref.kv_len])


def test_tree_oracle_rejects_a_parent_that_is_not_an_earlier_token():
    cfg = dict(SMALL, n_layers=1)
    layers = si.make_layers(cfg, seed=16)
    st = oracle.OracleStage(cfg, layers, 8)
    hidden = si.make_hidden(cfg, seed=16, n_tokens=3)
    for bad in ([-1, 1, 0], [-1, 0, 2], [-2, 0, 0], [0, 0, 0]):
        with pytest.raises(RuntimeError):
            st.prefill_tree(hidden, bad)
