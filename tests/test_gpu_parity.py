"""GPU parity: the HIP library against the CPU oracle, through the C ABI, on the same seeded inputs.

Bars: fp32 check mode max-abs <= 1e-3 and rel-L2 <= 1e-4; bf16 and 4-bit stages rel-L2 <= 2e-2 on hidden_out and on
the cached K/V values as whole tensors AND <= 4e-2 for every row by itself (one token's hidden state, one cached key
or value vector of one head; helpers.Pair.check does both); which cache slots are written, and nothing else, bit-exact.
"""
import numpy as np
import pytest

from helpers import BF16_REL_L2, Pair, rel_l2, to_numpy
from paper_2504_08242_amd import binding as jb
from paper_2504_08242_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def torch_mod():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def kv_bits(kv):
    torch = torch_mod()
    v = kv.view()
    return v.view(torch.int32 if kv.dtype == "f32" else torch.int16).cpu().numpy().copy()


def fill_sentinel(kv):
    torch = torch_mod()
    if kv.dtype == "f32":
        kv.buf.view(torch.int32).fill_(0x7FC12345)  # a NaN payload no kernel produces
    else:
        kv.buf.view(torch.int16).fill_(0x7FC1)
    torch.cuda.synchronize()


def assert_only_slots_changed(before, after, lo, hi, what=""):
    """Slots [lo, hi) of every (layer, K|V, head) changed, all others are bit-identical."""
    assert np.array_equal(before[:, :, :, :lo], after[:, :, :, :lo]), what
    assert np.array_equal(before[:, :, :, hi:], after[:, :, :, hi:]), what
    changed = before[:, :, :, lo:hi] != after[:, :, :, lo:hi]
    assert changed.all(), what  # sentinel is a NaN pattern: every written element differs


# ------------------------------------------------------------------------------------------------
# fp32 check mode
# ------------------------------------------------------------------------------------------------
def test_c1_tiny_stage_four_chunks_and_one_shot():
    """Config 1: 2 layers, d=256, 4x64 heads, FFN 688; 128 tokens as 4x32, and one shot."""
    p = Pair(si.TINY, "f32", seed=0, max_positions=128, max_chunk_tokens=128)
    hidden = p.hidden(128)
    g4, o4 = p.run_both(hidden, [32, 32, 32, 32])
    p.check(g4, o4, "4x32")
    kv4 = p.kv_gpu()
    p.check(kv4, p.oracle.kv, "kv 4x32")
    g1, o1 = p.run_both(hidden, [128])
    p.check(g1, o1, "1x128")
    p.check(g1, o4, "one-shot vs chunked oracle")
    p.check(g4, g1, "chunked vs one-shot on the GPU")
    p.check(p.kv_gpu(), kv4, "kv one-shot vs chunked")


def test_f32_ragged_chunks_write_exactly_their_cache_slots():
    cfg = dict(si.TINY, n_layers=3)
    p = Pair(cfg, "f32", seed=5, max_positions=140, max_chunk_tokens=70, weight_std=1.0 / 16.0)
    hidden = p.hidden(131)
    fill_sentinel(p.kv)
    pos, outs = 0, []
    for n in [1, 5, 37, 64, 3, 21]:
        before = kv_bits(p.kv)
        g = p.gpu_chunk(hidden[pos:pos + n], pos)
        after = kv_bits(p.kv)
        assert_only_slots_changed(before, after, pos, pos + n, f"chunk at {pos}")
        o = p.oracle.prefill_chunk(hidden[pos:pos + n], pos)
        p.check(g, o, f"chunk at {pos}")
        pos += n
        assert len(p.kv) == pos
    p.check(p.kv_gpu()[:, :, :, :pos], p.oracle.kv[:, :, :, :pos], "kv")


def test_f32_odd_shapes():
    cfg = dict(n_layers=2, d_model=120, n_heads=3, head_dim=40, d_ffn=172, rms_eps=1e-6, rope_theta=500.0)
    p = Pair(cfg, "f32", seed=8, max_positions=40, max_chunk_tokens=33, weight_std=0.09)
    hidden = p.hidden(40)
    g, o = p.run_both(hidden, [33, 7])
    p.check(g, o)
    p.check(p.kv_gpu(), p.oracle.kv, "kv")


def test_f32_zero_output_projections_pass_input_through_bitwise():
    cfg = si.TINY
    layers = si.make_layers(cfg, seed=2)
    for w in layers:
        w["wo"] = np.zeros_like(w["wo"])
        w["w_down"] = np.zeros_like(w["w_down"])
    p = Pair(cfg, "f32", seed=2, max_positions=16, max_chunk_tokens=16, layers_np=layers)
    hidden = p.hidden(16)
    g = p.gpu_chunk(hidden, 0)
    assert np.array_equal(g, hidden)


def test_error_codes_through_prefill_and_cache_length_bookkeeping():
    torch = torch_mod()
    p = Pair(si.TINY, "f32", seed=1, max_positions=48, max_chunk_tokens=32)
    x = torch.from_numpy(p.hidden(32)).cuda()
    st, kv = p.stage, p.kv
    with pytest.raises(jb.JupiterError) as e:
        st.prefill_chunk(x, 1, kv)  # hole
    assert e.value.status == jb.JUP_EPOS and len(kv) == 0
    st.prefill_chunk(x, 0, kv)
    assert len(kv) == 32
    with pytest.raises(jb.JupiterError) as e:
        st.prefill_chunk(x, 32, kv)  # 32 + 32 > 48
    assert e.value.status == jb.JUP_ECAP and len(kv) == 32
    with pytest.raises(jb.JupiterError) as e:
        st.prefill_chunk(torch.zeros(33, 256, device="cuda"), 0, kv)  # above max_chunk_tokens
    assert e.value.status == jb.JUP_ECAP
    st.prefill_chunk(x[:0], 32, kv)  # empty chunk: no-op
    assert len(kv) == 32
    st.prefill_chunk(x[:16], 16, kv)  # overwrite from 16: implicit truncate
    assert len(kv) == 32
    st.prefill_chunk(x[:4], 8, kv)
    assert len(kv) == 12
    other = jb.KvCache(dict(si.TINY, n_heads=2, head_dim=128), "f32", 48)
    with pytest.raises(jb.JupiterError) as e:
        st.prefill_chunk(x, 0, other)
    assert e.value.status == jb.JUP_EINVAL
    torch.cuda.synchronize()


def test_f32_hidden_out_may_alias_hidden_in():
    torch = torch_mod()
    p = Pair(si.TINY, "f32", seed=3, max_positions=24, max_chunk_tokens=24)
    h = p.hidden(24)
    want = p.gpu_chunk(h, 0)
    p.kv.reset()
    x = torch.from_numpy(h).cuda()
    p.stage.prefill_chunk(x, 0, p.kv, hidden_out=x)
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(x), want)


def test_f32_truncate_after_rejected_candidates_equals_never_appending_them():
    """Speculative verification (Sec. V-A steps 3 and 5): candidates are cached, the rejected ones removed."""
    p = Pair(si.TINY, "f32", seed=4, max_positions=64, max_chunk_tokens=32)
    h = p.hidden(40)
    cand = p.hidden(5, tag=1)
    p.gpu_chunk(h[:20], 0)
    p.gpu_chunk(cand, 20)          # 1 token + 4 drafts
    p.kv.truncate(22)              # two accepted
    a = p.gpu_chunk(h[20:30], 22)
    kv_a = kv_bits(p.kv)[:, :, :, :32]
    p.kv.reset()
    p.gpu_chunk(h[:20], 0)
    p.gpu_chunk(cand[:2], 20)
    b = p.gpu_chunk(h[20:30], 22)
    assert np.array_equal(a, b)
    assert np.array_equal(kv_a, kv_bits(p.kv)[:, :, :, :32])


# ------------------------------------------------------------------------------------------------
# token tree of a speculative step (Sec. V-A): candidates verified in one call, rejected ones removed
# ------------------------------------------------------------------------------------------------
def tree_paths(parents):
    paths = []
    for t, par in enumerate(parents):
        paths.append((paths[par] if par >= 0 else []) + [t])
    return paths


def run_tree_case(p, n_prefix, n_tree, seed, n_after=7):
    """Prefix, then a token tree, then keep the deepest path and go on: GPU against the oracle at every step."""
    parents = si.make_token_tree(n_tree, seed)
    paths = tree_paths(parents)
    h = p.hidden(n_prefix + n_tree + n_after)
    pre, cand, after = h[:n_prefix], h[n_prefix:n_prefix + n_tree], h[n_prefix + n_tree:]
    p.kv.reset(); p.oracle.reset()
    fill_sentinel(p.kv)
    if n_prefix:
        p.gpu_chunk(pre, 0)
        p.oracle.prefill_chunk(pre, 0)
    before = kv_bits(p.kv)
    g = p.gpu_tree(cand, n_prefix, parents)
    o = p.oracle.prefill_tree(cand, parents, n_prefix)
    p.check(g, o, "tree output")
    assert len(p.kv) == n_prefix + n_tree
    after_bits = kv_bits(p.kv)
    assert_only_slots_changed(before, after_bits, n_prefix, n_prefix + n_tree, "tree slots")
    p.check(p.kv_gpu()[:, :, :, :n_prefix + n_tree], p.oracle.kv[:, :, :, :n_prefix + n_tree], "tree cache")

    # accept the deepest path; the kept entries are moved bit for bit, everything below base stays
    path = max(paths, key=len)
    assert len(path) >= 3 and path != list(range(len(path))), "the case must move entries"
    p.kv.keep(n_prefix, path)
    p.oracle.keep(n_prefix, path)
    assert len(p.kv) == n_prefix + len(path) == p.oracle.kv_len
    kept = kv_bits(p.kv)
    assert np.array_equal(kept[:, :, :, :n_prefix], after_bits[:, :, :, :n_prefix])
    for j, t in enumerate(path):
        assert np.array_equal(kept[:, :, :, n_prefix + j], after_bits[:, :, :, n_prefix + t]), (j, t)
    # ... and the sequence continues as if only the accepted tokens had ever been fed
    g2 = p.gpu_chunk(after, len(p.kv))
    o2 = p.oracle.prefill_chunk(after, p.oracle.kv_len)
    p.check(g2, o2, "chunk after keep")
    return parents, paths, cand, g


def test_f32_token_tree_matches_the_oracle_and_keep_moves_the_accepted_path():
    p = Pair(si.TINY, "f32", seed=21, max_positions=128, max_chunk_tokens=64)
    run_tree_case(p, n_prefix=37, n_tree=64, seed=21)
    run_tree_case(p, n_prefix=0, n_tree=11, seed=22)


def test_f32_tree_node_equals_the_ordinary_call_on_its_path():
    """The property verification relies on, on the GPU alone: row t = last row of the chain call on t's path."""
    p = Pair(si.TINY, "f32", seed=23, max_positions=96, max_chunk_tokens=64)
    n_prefix, n_tree = 19, 24
    parents = si.make_token_tree(n_tree, 23)
    h = p.hidden(n_prefix + n_tree)
    p.gpu_chunk(h[:n_prefix], 0)
    g = p.gpu_tree(h[n_prefix:], n_prefix, parents)
    for t, path in enumerate(tree_paths(parents)):
        if t % 5 and len(path) < 4:
            continue
        p.kv.truncate(n_prefix)
        ref = p.gpu_chunk(h[n_prefix:][path], n_prefix)
        assert np.max(np.abs(g[t] - ref[-1])) <= 2e-5, t   # same arithmetic, other kernel shapes and orders


def test_f32_chain_shaped_tree_is_bitwise_the_ordinary_chunk():
    p = Pair(si.TINY, "f32", seed=24, max_positions=64, max_chunk_tokens=64)
    h = p.hidden(50)
    p.gpu_chunk(h[:10], 0)
    a = p.gpu_chunk(h[10:], 10)
    kv_a = kv_bits(p.kv)
    p.kv.truncate(10)
    b = p.gpu_tree(h[10:], 10, list(range(-1, 39)))
    assert np.array_equal(a, b)
    assert np.array_equal(kv_a, kv_bits(p.kv))


def test_tree_and_keep_argument_errors_leave_the_cache_untouched():
    p = Pair(si.TINY, "f32", seed=25, max_positions=80, max_chunk_tokens=80)
    h = p.hidden(70)
    p.gpu_chunk(h[:8], 0)
    E = jb.JupiterError
    for parents, status in (([-1, 1, 0], jb.JUP_EINVAL), ([0, 0, 0], jb.JUP_EINVAL), ([-2, 0, 1], jb.JUP_EINVAL)):
        with pytest.raises(E) as ei:
            p.gpu_tree(h[8:11], 8, parents)
        assert ei.value.status == status and len(p.kv) == 8
    with pytest.raises(E) as ei:                      # more than the 64 tokens of a tree
        p.gpu_tree(h[:65], 8, list(range(-1, 64)))
    assert ei.value.status == jb.JUP_EINVAL and len(p.kv) == 8
    with pytest.raises(E) as ei:                      # a hole
        p.gpu_tree(h[8:11], 9, [-1, 0, 1])
    assert ei.value.status == jb.JUP_EPOS
    p.gpu_tree(h[8:14], 8, [-1, 0, 0, 1, 1, 2])
    assert len(p.kv) == 14
    for base, slots, status in ((8, [1, 0], jb.JUP_EINVAL), (8, [0, 0], jb.JUP_EINVAL), (8, [-1], jb.JUP_EINVAL),
                                (8, [0, 6], jb.JUP_EPOS), (15, [], jb.JUP_EPOS), (-1, [], jb.JUP_EPOS)):
        with pytest.raises(E) as ei:
            p.kv.keep(base, slots)
        assert ei.value.status == status and len(p.kv) == 14, (base, slots)
    p.kv.keep(8, [0, 2, 5])
    assert len(p.kv) == 11
    p.kv.keep(8, [])                                   # all candidates rejected = truncate
    assert len(p.kv) == 8


def test_keep_on_a_fork_moves_only_the_forks_own_entries():
    p = Pair(si.TINY, "f32", seed=26, max_positions=64, max_chunk_tokens=64)
    h = p.hidden(40)
    p.gpu_chunk(h[:16], 0)
    parent_bits = kv_bits(p.kv)
    fork = p.kv.fork(16, 48)
    fill_sentinel(fork)
    p.gpu_chunk(h[16:20], 16, kv=fork)
    p.gpu_tree(h[20:30], 20, [-1, 0, 0, 1, 1, 2, 3, 3, 6, 8], kv=fork)
    before = kv_bits(fork)
    with pytest.raises(jb.JupiterError) as ei:
        fork.keep(15, [0])                             # inside the shared prefix
    assert ei.value.status == jb.JUP_EPOS
    fork.keep(20, [0, 1, 3, 6, 8])
    after = kv_bits(fork)
    assert len(fork) == 25
    assert np.array_equal(kv_bits(p.kv), parent_bits)
    assert np.array_equal(after[:, :, :, :4], before[:, :, :, :4])           # own slots of positions 16..19
    for j, t in enumerate([0, 1, 3, 6, 8]):
        assert np.array_equal(after[:, :, :, 4 + j], before[:, :, :, 4 + t])
    fork.destroy()


def run_fork_case(p, n_prefix, n_private, n_chunk, n_branches):
    """Shared prompt prefix, per-branch private tokens, then one small chunk per branch (Sec. V-B)."""
    cfg = p.cfg
    prefix = p.hidden(n_prefix)
    p.kv.reset()
    p.oracle.reset()
    pos = 0
    step = p.stage.max_chunk_tokens
    while pos < n_prefix:  # prefill the shared prompt on both sides
        n = min(step, n_prefix - pos)
        p.gpu_chunk(prefix[pos:pos + n], pos)
        p.oracle.prefill_chunk(prefix[pos:pos + n], pos)
        pos += n
    parent_bits = kv_bits(p.kv)
    oracle_prefix_kv = p.oracle.kv.copy()
    forks = [p.kv.fork(n_prefix, n_prefix + n_private + n_chunk) for _ in range(n_branches)]
    for b, fk in enumerate(forks):
        assert len(fk) == n_prefix
        priv = p.hidden(n_private, tag=100 + b)
        chunk = p.hidden(n_chunk, tag=200 + b)
        p.oracle.kv[...] = oracle_prefix_kv  # the oracle works on an unshared copy of the prefix
        o_priv = p.oracle.prefill_chunk(priv, n_prefix)
        o_chunk = p.oracle.prefill_chunk(chunk, n_prefix + n_private)
        g_priv = p.gpu_chunk(priv, n_prefix, kv=fk)
        g_chunk = p.gpu_chunk(chunk, n_prefix + n_private, kv=fk)
        p.check(g_priv, o_priv, f"branch {b} private tokens")
        p.check(g_chunk, o_chunk, f"branch {b} chunk")
        assert len(fk) == n_prefix + n_private + n_chunk
        own = to_numpy(fk.view())
        p.check(own, p.oracle.kv[:, :, :, n_prefix:n_prefix + n_private + n_chunk], f"branch {b} private kv")
        assert np.array_equal(p.oracle.kv[:, :, :, :n_prefix], oracle_prefix_kv[:, :, :, :n_prefix])
        with pytest.raises(jb.JupiterError) as e:
            p.stage.prefill_chunk(p_tensor(p, chunk), n_prefix - 1, fk)  # inside the shared prefix
        assert e.value.status == jb.JUP_EPOS
    assert np.array_equal(parent_bits, kv_bits(p.kv))  # the shared prefix was only read
    with pytest.raises(jb.JupiterError) as e:
        p.kv.truncate(n_prefix - 1)  # forks still share it
    assert e.value.status == jb.JUP_EPOS
    for fk in forks:
        fk.destroy()
    p.kv.truncate(n_prefix - 1)


def run_batched_branches_case(p, n_prefix, n_privates, n_chunk, exact=True, close=4e-3):
    """All branches advance by n_chunk tokens in ONE call; the result must equal one call per branch bit for
    bit (outputs and caches), and the oracle within tolerance.  exact=False: the batched rows run other projection
    kernels than a single branch's: equal within `close` (rel-L2) instead; the oracle check is the same either way."""
    torch = torch_mod()
    nb = len(n_privates)
    prefix = p.hidden(n_prefix)
    p.kv.reset()
    p.oracle.reset()
    step = p.stage.max_chunk_tokens
    for pos in range(0, n_prefix, step):
        n = min(step, n_prefix - pos)
        p.gpu_chunk(prefix[pos:pos + n], pos)
        p.oracle.prefill_chunk(prefix[pos:pos + n], pos)
    oracle_prefix_kv = p.oracle.kv.copy()
    cap = n_prefix + max(n_privates) + n_chunk
    forks = [p.kv.fork(n_prefix, cap) for _ in range(nb)]
    chunks = [p.hidden(n_chunk, tag=200 + b) for b in range(nb)]
    seq_out, seq_kv, ora_out = [], [], []
    for b, fk in enumerate(forks):
        priv = p.hidden(n_privates[b], tag=100 + b)
        p.oracle.kv[...] = oracle_prefix_kv
        p.oracle.prefill_chunk(priv, n_prefix)
        ora_out.append(p.oracle.prefill_chunk(chunks[b], n_prefix + n_privates[b]))
        p.gpu_chunk(priv, n_prefix, kv=fk)
        seq_out.append(p.gpu_chunk(chunks[b], n_prefix + n_privates[b], kv=fk))
        seq_kv.append(kv_bits(fk).copy())
    # again, all branches in one call; the chunk of the sequential pass is overwritten (pos_offset < length)
    x = torch.from_numpy(np.concatenate(chunks)).to(device="cuda:0", dtype=p.td)
    pos = [n_prefix + n for n in n_privates]
    # poison the slots the batched call must rewrite, so that equality below proves they were written
    for b, fk in enumerate(forks):
        fk.view()[:, :, :, n_privates[b]:n_privates[b] + n_chunk, :] = 7.0
    y = to_numpy(p.stage.prefill_branches(x, n_chunk, pos, forks))
    torch.cuda.synchronize()
    for b, fk in enumerate(forks):
        got = y[b * n_chunk:(b + 1) * n_chunk]
        if exact:
            assert np.array_equal(got, seq_out[b]), f"branch {b}: batched output differs from the per-branch call"
            assert np.array_equal(kv_bits(fk), seq_kv[b]), f"branch {b}: batched cache differs"
        else:
            assert rel_l2(got, seq_out[b]) <= close, (b, rel_l2(got, seq_out[b]))
            now, before = kv_bits(fk), seq_kv[b]
            lo, hi = n_privates[b], n_privates[b] + n_chunk  # the chunk's slots in the fork's own buffer
            rewritten = np.zeros(now.shape, bool)
            rewritten[..., lo:hi, :] = True
            assert np.array_equal(now[~rewritten], before[~rewritten]), f"branch {b}: other cache slots written"
            as_f32 = lambda bits: (bits.astype(np.uint16).astype(np.uint32) << 16).view(np.float32)
            assert rel_l2(as_f32(now[..., lo:hi, :]), as_f32(before[..., lo:hi, :])) <= close
        p.check(got, ora_out[b], f"branch {b} chunk (batched)")
        assert len(fk) == pos[b] + n_chunk
    # validation happens before anything is enqueued and leaves every cache as it was
    lens = [len(fk) for fk in forks]
    for bad_kvs, bad_pos, status in (
            ([forks[0], forks[0]], [pos[0], pos[0]], jb.JUP_EINVAL),          # the same cache twice
            ([p.kv, forks[0]], [n_prefix, pos[0]], jb.JUP_EINVAL),           # parent and fork together
            ([forks[0], forks[1]], [pos[0], lens[1] + 1], jb.JUP_EPOS),      # a hole in the second branch
            ([forks[0], forks[1]], [pos[0], n_prefix - 1], jb.JUP_EPOS)):    # inside the shared prefix
        with pytest.raises(jb.JupiterError) as e:
            p.stage.prefill_branches(x[:2 * n_chunk], n_chunk, bad_pos, bad_kvs)
        assert e.value.status == status
        assert [len(fk) for fk in forks] == lens
    with pytest.raises(jb.JupiterError) as e:  # more rows than the stage's workspace holds
        big = torch.zeros((nb * (step // nb + 1), p.cfg["d_model"]), device="cuda:0", dtype=p.td)
        p.stage.prefill_branches(big, step // nb + 1, pos, forks)
    assert e.value.status == jb.JUP_ECAP
    for fk in forks:
        fk.destroy()


def test_f32_batched_branches_equal_one_call_per_branch():
    p = Pair(si.TINY, "f32", seed=8, max_positions=40, max_chunk_tokens=16, oracle_positions=64)
    run_batched_branches_case(p, n_prefix=37, n_privates=[9, 4, 12], n_chunk=5)


def test_bf16_batched_branches_equal_one_call_per_branch_bitwise():
    """Outline branches advanced together (Sec. V-B): the weights are streamed once for all of them."""
    cfg = dict(si.LLAMA7B_STAGE, n_layers=2)
    p = Pair(cfg, "bf16", seed=9, max_positions=72, max_chunk_tokens=64, oracle_positions=128)
    run_batched_branches_case(p, n_prefix=70, n_privates=[9, 33, 12, 1], n_chunk=5)


def p_tensor(p, a):
    torch = torch_mod()
    return torch.from_numpy(a).to(device="cuda:0", dtype=p.td)


def test_f32_forked_caches_share_the_prompt_prefix():
    p = Pair(si.TINY, "f32", seed=6, max_positions=40, max_chunk_tokens=16, oracle_positions=51)
    run_fork_case(p, n_prefix=37, n_private=9, n_chunk=5, n_branches=3)


def test_same_call_twice_is_bitwise_identical():
    p = Pair(si.TINY, "f32", seed=7, max_positions=64, max_chunk_tokens=64)
    h = p.hidden(64)
    a = p.gpu_chunk(h, 0)
    p.kv.reset()
    b = p.gpu_chunk(h, 0)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------------------------------------
# bf16 matrix-core path
# ------------------------------------------------------------------------------------------------
LLAMA7B_2L = dict(si.LLAMA7B_STAGE, n_layers=2)


def test_bf16_two_layer_7b_shape_ragged_chunks_and_cache_slots():
    p = Pair(LLAMA7B_2L, "bf16", seed=11, max_positions=300, max_chunk_tokens=128)
    hidden = p.hidden(277)
    fill_sentinel(p.kv)
    pos = 0
    for n in [64, 37, 5, 128, 1, 42]:
        before = kv_bits(p.kv)
        g = p.gpu_chunk(hidden[pos:pos + n], pos)
        after = kv_bits(p.kv)
        assert_only_slots_changed(before, after, pos, pos + n, f"chunk at {pos}")
        o = p.oracle.prefill_chunk(hidden[pos:pos + n], pos)
        p.check(g, o, f"chunk at {pos}")
        pos += n
    kv = p.kv_gpu()[:, :, :, :pos]
    for l in range(2):
        for which in range(2):
            p.check(kv[l, which], p.oracle.kv[l, which, :, :pos], f"cache layer {l} {'KV'[which]}")


def test_bf16_layer0_cache_is_bit_identical_across_chunkings_and_runs():
    """K and V of the first layer are row-local functions of the input: chunking must not change a bit."""
    p = Pair(LLAMA7B_2L, "bf16", seed=12, max_positions=256, max_chunk_tokens=256)
    hidden = p.hidden(256)
    outs, kvs = [], []
    for chunks in ([256], [64, 64, 64, 64], [100, 29, 127], [256]):
        p.kv.reset()
        pos, g = 0, []
        for n in chunks:
            g.append(p.gpu_chunk(hidden[pos:pos + n], pos))
            pos += n
        outs.append(np.concatenate(g))
        kvs.append(kv_bits(p.kv))
    assert np.array_equal(outs[0], outs[3]) and np.array_equal(kvs[0], kvs[3])  # same call twice
    for i in (1, 2):
        assert np.array_equal(kvs[0][0], kvs[i][0]), "layer-0 cache differs between chunkings"
        assert rel_l2(outs[i], outs[0]) <= BF16_REL_L2


def test_bf16_forked_caches_share_the_prompt_prefix_small():
    p = Pair(LLAMA7B_2L, "bf16", seed=13, max_positions=80, max_chunk_tokens=64, oracle_positions=86)
    run_fork_case(p, n_prefix=70, n_private=11, n_chunk=5, n_branches=2)


def test_bf16_token_tree_matches_the_oracle_and_keep_moves_the_accepted_path():
    p = Pair(LLAMA7B_2L, "bf16", seed=31, max_positions=200, max_chunk_tokens=128)
    run_tree_case(p, n_prefix=100, n_tree=64, seed=31)     # tree entries span the tiles 3..5 of 32 keys
    run_tree_case(p, n_prefix=37, n_tree=26, seed=32)      # one query block, ragged
    run_tree_case(p, n_prefix=0, n_tree=40, seed=33)


def test_bf16_chain_shaped_tree_is_bitwise_the_ordinary_chunk():
    p = Pair(LLAMA7B_2L, "bf16", seed=34, max_positions=128, max_chunk_tokens=64)
    h = p.hidden(90)
    p.gpu_chunk(h[:41], 0)
    a = p.gpu_chunk(h[41:], 41)
    kv_a = kv_bits(p.kv)
    p.kv.truncate(41)
    b = p.gpu_tree(h[41:], 41, list(range(-1, 48)))
    assert np.array_equal(a, b)
    assert np.array_equal(kv_a, kv_bits(p.kv))


def test_bf16_tree_node_equals_the_ordinary_call_on_its_path():
    p = Pair(LLAMA7B_2L, "bf16", seed=35, max_positions=128, max_chunk_tokens=128)
    n_prefix, n_tree = 70, 48
    parents = si.make_token_tree(n_tree, 35)
    h = p.hidden(n_prefix + n_tree)
    p.gpu_chunk(h[:n_prefix], 0)
    g = p.gpu_tree(h[n_prefix:], n_prefix, parents)
    for t, path in enumerate(tree_paths(parents)):
        if t % 7:
            continue
        p.kv.truncate(n_prefix)
        ref = p.gpu_chunk(h[n_prefix:][path], n_prefix)
        assert rel_l2(g[t], ref[-1]) <= 1e-2, t   # same values, other tile shapes and summation orders


def test_bf16_short_chunks_behind_a_long_cache_split_their_keys_over_workgroups():
    """Chunks of up to 256 tokens behind 1000+ cached positions: the key tiles of a query block are split over several
    workgroups and merged by the last one to finish (decoding steps of Sec. V against a long sequence).  Against the
    oracle row by row, and twice: the merge order is fixed, so the bits must not depend on which workgroup came last."""
    p = Pair(LLAMA7B_2L, "bf16", seed=15, max_positions=1600, max_chunk_tokens=300)
    sizes = [5, 1, 37, 64, 100, 200, 31]          # 1-2 query blocks of 32, then 64-query blocks with 2 or 4 key ranges
    hidden = p.hidden(1100 + sum(sizes) + 26)
    p.run_both(hidden[:1100], [275] * 4)
    pos = 1100
    for n in sizes:
        h = hidden[pos:pos + n]
        want = p.oracle.prefill_chunk(h, pos)
        got = p.gpu_chunk(h, pos)
        p.check(got, want, f"chunk of {n} at {pos}")
        bits = kv_bits(p.kv)
        for rep in range(3):
            assert np.array_equal(p.gpu_chunk(h, pos), got), (n, rep)      # pos < length: overwrite from there
            assert np.array_equal(kv_bits(p.kv), bits), (n, rep)
        pos += n
    parents = si.make_token_tree(26, 15)
    h = hidden[pos:pos + 26]
    got = p.gpu_tree(h, pos, parents)
    p.check(got, p.oracle.prefill_tree(h, parents, pos), f"tree at {pos}")
    p.kv.truncate(pos)
    assert np.array_equal(p.gpu_tree(h, pos, parents), got)
    kv = p.kv_gpu()[:, :, :, :pos + 26]
    for l in range(2):
        p.check(kv[l], p.oracle.kv[l, :, :, :pos + 26], f"cache layer {l}")
    # a chain-shaped tree is the ordinary chunk, bit for bit, with split keys too
    p.kv.truncate(pos)
    a = p.gpu_chunk(h, pos)
    p.kv.truncate(pos)
    assert np.array_equal(p.gpu_tree(h, pos, list(range(-1, 25))), a)


def test_bf16_batched_branches_with_split_keys_equal_one_call_per_branch_bitwise():
    """Branches whose caches straddle the length at which a query block gets a second key range: alone or batched, a
    branch takes the same ranges and merges them in the same order."""
    p = Pair(LLAMA7B_2L, "bf16", seed=16, max_positions=975, max_chunk_tokens=325, oracle_positions=1100)
    run_batched_branches_case(p, n_prefix=975, n_privates=[9, 33, 12, 1], n_chunk=5)   # 989, 1013, 992, 981 keys


def assert_same_cache_entries(got_bits, want_bits, sentinel_bits):
    """The same entries were written (everything else still holds the sentinel), whatever their values."""
    assert np.array_equal(got_bits == sentinel_bits, want_bits == sentinel_bits)


def run_chunks_case(p, chunks, pos0_chunks=(), exact=True):
    """jup_stage_prefill_chunks against one call per chunk: outputs, cache and length.  Bit for bit when the chunks
    run one after the other; up to fp32 summation order (fewer K splits) when they overlap."""
    import torch
    total = sum(pos0_chunks) + sum(chunks)
    h = p.hidden(total)
    def prefix():
        p.kv.reset()
        fill_sentinel(p.kv)
        pos = 0
        for n in pos0_chunks:
            p.gpu_chunk(h[pos:pos + n], pos)
            pos += n
        return pos
    pos0 = prefix()
    want, pos = [], pos0
    for n in chunks:
        want.append(p.gpu_chunk(h[pos:pos + n], pos))
        pos += n
    want = np.concatenate(want) if want else np.zeros((0, p.cfg["d_model"]), np.float32)
    kv_want, kvv_want, len_want = kv_bits(p.kv), p.kv_gpu(), len(p.kv)
    prefix()
    x = torch.from_numpy(h[pos0:]).to(device="cuda:0", dtype=p.td)
    y = to_numpy(p.stage.prefill_chunks(x, chunks, pos0, p.kv))
    torch.cuda.synchronize()
    assert len(p.kv) == len_want
    if exact:
        assert np.array_equal(y, want)
        assert np.array_equal(kv_bits(p.kv), kv_want)
    else:
        sentinel = np.int32(0x7FC12345) if p.dtype == "f32" else np.int16(0x7FC1)
        assert_same_cache_entries(kv_bits(p.kv), kv_want, sentinel)
        if len(want):
            assert rel_l2(y, want) <= 4e-3, rel_l2(y, want)      # bf16 last-bit differences after two layers
            live = kv_want != sentinel
            assert rel_l2(p.kv_gpu()[live], kvv_want[live]) <= 4e-3
        # deterministic: the same call again gives the same bits
        bits1 = kv_bits(p.kv)
        prefix()
        y2 = to_numpy(p.stage.prefill_chunks(x, chunks, pos0, p.kv))
        assert np.array_equal(y2, y) and np.array_equal(kv_bits(p.kv), bits1)
    return y, h[pos0:]


@pytest.mark.parametrize("n_lanes", [2, 3, 4])
def test_bf16_overlapped_chunks_equal_one_call_per_chunk(n_lanes):
    """Consecutive chunks on several streams: a chunk may only read what the chunks before it have already cached.
    A missing dependency would show as a mismatch far above rounding, or as a run-to-run difference."""
    p = Pair(LLAMA7B_2L, "bf16", seed=41, max_positions=700, max_chunk_tokens=192)
    run_chunks_case(p, [64, 64, 64])                       # not enabled yet: one after the other
    p.stage.enable_overlap(n_lanes)
    for rep in range(3):                                    # repeated: a missing dependency shows as a flaky mismatch
        run_chunks_case(p, [128, 37, 0, 5, 192, 64, 1, 100], pos0_chunks=[50], exact=False)
    got, h = run_chunks_case(p, [160, 160, 160, 160], exact=False)
    o = [p.oracle.prefill_chunk(h[i * 160:(i + 1) * 160], i * 160) for i in range(4)]
    p.check(got, np.concatenate(o), "overlapped chunks vs oracle")
    run_chunks_case(p, [96])                                # a single chunk takes the plain path
    run_chunks_case(p, [])


def test_prefill_chunks_argument_errors_and_check_mode():
    p = Pair(si.TINY, "f32", seed=42, max_positions=64, max_chunk_tokens=32)
    run_chunks_case(p, [32, 7, 0, 20])                      # check mode: sequential, same results
    import torch
    x = torch.zeros((40, p.cfg["d_model"]), device="cuda:0", dtype=p.td)
    p.kv.reset()
    for chunks, status in (([33, 7], jb.JUP_ECAP), ([32, -1, 9], jb.JUP_EINVAL)):
        with pytest.raises(jb.JupiterError) as ei:
            p.stage.prefill_chunks(x[:sum(max(c, 0) for c in chunks)], chunks, 0, p.kv)
        assert ei.value.status == status and len(p.kv) == 0
    with pytest.raises(jb.JupiterError) as ei:              # the chunks together overflow the cache
        p.stage.prefill_chunks(torch.zeros((70, p.cfg["d_model"]), device="cuda:0", dtype=p.td), [30, 30, 10], 0, p.kv)
    assert ei.value.status == jb.JUP_ECAP and len(p.kv) == 0
    with pytest.raises(jb.JupiterError) as ei:              # a hole before the first chunk
        p.stage.prefill_chunks(x[:10], [10], 3, p.kv)
    assert ei.value.status == jb.JUP_EPOS
    for bad in (1, 5):
        with pytest.raises(jb.JupiterError) as ei:
            p.stage.enable_overlap(bad)
        assert ei.value.status == jb.JUP_EINVAL
    with pytest.raises(jb.JupiterError):                    # accepted once (check mode then still runs the chunks in turn)
        p.stage.enable_overlap(2); p.stage.enable_overlap(2)  # twice is an error


def test_bf16_zero_output_projections_pass_input_through_bitwise():
    cfg = LLAMA7B_2L
    layers = si.make_layers(cfg, seed=14, bf16=True)
    for w in layers:
        w["wo"] = np.zeros_like(w["wo"])
        w["w_down"] = np.zeros_like(w["w_down"])
    p = Pair(cfg, "bf16", seed=14, max_positions=70, max_chunk_tokens=70, layers_np=layers)
    hidden = p.hidden(70)
    assert np.array_equal(p.gpu_chunk(hidden, 0), hidden)
    # rows are read 16 bytes at a time: a hidden-state pointer off by one element is refused on the host
    torch = torch_mod()
    flat = torch.zeros(4 * cfg["d_model"] + 1, device="cuda:0", dtype=torch.bfloat16)
    with pytest.raises(jb.JupiterError) as e:
        p.stage.prefill_chunk(flat[1:].view(4, cfg["d_model"]), 0, p.kv)
    assert e.value.status == jb.JUP_EINVAL and "aligned" in str(e.value) and len(p.kv) == 70


@pytest.mark.parametrize("d_model,n_heads,d_ffn,n_layers", [(256, 2, 128, 3), (768, 6, 896, 2), (1536, 12, 4224, 2)])
def test_bf16_small_and_odd_stage_shapes(d_model, n_heads, d_ffn, n_layers):
    """The smallest widths the bf16 path accepts and widths that are no power of two: K loops of one to a few stages
    per workgroup, tiles wider than the matrix, the generic reduce + norm, every row-tile height (chunks of 5 to 200
    tokens), a token tree and an overlapped multi-chunk call."""
    import torch
    cfg = dict(si.LLAMA7B_STAGE, d_model=d_model, n_heads=n_heads, d_ffn=d_ffn, n_layers=n_layers)
    p = Pair(cfg, "bf16", seed=70 + n_heads, max_positions=900, max_chunk_tokens=200)
    chunks = [5, 64, 100, 200, 31]
    hidden = p.hidden(sum(chunks) + 26 + 401)
    g, o = p.run_both(hidden, chunks)
    p.check(g, o, "chunk by chunk")
    row = 0
    for n in chunks:
        p.check(g[row:row + n], o[row:row + n], f"chunk of {n} at {row}")
        row += n
    parents = si.make_token_tree(26, 70)
    h = hidden[row:row + 26]
    p.check(p.gpu_tree(h, row, parents), p.oracle.prefill_tree(h, parents, row), "tree")
    row += 26
    kv = p.kv_gpu()[:, :, :, :row]
    for l in range(n_layers):
        p.check(kv[l], p.oracle.kv[l, :, :, :row], f"cache layer {l}")
    # the same prompt prefix again plus more, in one overlapped call behind the tree
    more = [100, 200, 37, 64]
    p.stage.enable_overlap(4)
    x = torch.from_numpy(hidden[row:row + sum(more)]).to(device="cuda:0", dtype=p.td)
    y = to_numpy(p.stage.prefill_chunks(x, more, row, p.kv))
    want, pos = [], row
    for n in more:
        want.append(p.oracle.prefill_chunk(hidden[pos:pos + n], pos))
        pos += n
    p.check(y, np.concatenate(want), "overlapped call")
    assert len(p.kv) == pos


@pytest.mark.parametrize("dtype", ["bf16", "w4"])
def test_decode_sized_call_captured_in_a_graph_replays_bit_identically(dtype):
    """A call enqueues kernels only (its tables travel as kernel arguments), so it can be captured in a HIP graph.
    Every replay, with eager work of the same stage between the replays, must give the eager call's bits."""
    torch = torch_mod()
    p = Pair(LLAMA7B_2L, dtype, seed=98, max_positions=128, max_chunk_tokens=64)
    h = p.hidden(64 + 5 + 5)
    p.gpu_chunk(h[:64], 0)
    x = torch.from_numpy(h[64:69]).to(device="cuda:0", dtype=p.td)
    other = torch.from_numpy(h[69:74]).to(device="cuda:0", dtype=p.td)
    y = torch.empty_like(x)
    p.stage.prefill_chunk(x, 64, p.kv, hidden_out=y)
    torch.cuda.synchronize()
    want, want_kv = y.clone(), kv_bits(p.kv)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        p.stage.prefill_chunk(x, 64, p.kv, hidden_out=y)
    torch.cuda.synchronize()
    for rep in range(3):
        # eager work in between: another chunk at the same position overwrites the slots and the scratch buffers
        p.stage.prefill_chunk(other, 64, p.kv)
        y.zero_()
        torch.cuda.synchronize()
        assert not np.array_equal(kv_bits(p.kv), want_kv)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), rep
        assert np.array_equal(kv_bits(p.kv), want_kv), rep


def test_c2_7b_stage_512_tokens_in_8_chunks_of_64():
    """Config 2: 8 layers of Llama-2-7B shape, bf16, 512-token prompt as 8 chunks of 64."""
    p = Pair(si.LLAMA7B_STAGE, "bf16", seed=20, max_positions=512, max_chunk_tokens=64)
    hidden = p.hidden(512)
    g, o = p.run_both(hidden, [64] * 8)
    p.check(g, o, "hidden_out")
    for c in range(8):
        p.check(g[c * 64:(c + 1) * 64], o[c * 64:(c + 1) * 64], f"chunk {c}")
    kv = p.kv_gpu()
    for l in range(8):
        p.check(kv[l], p.oracle.kv[l], f"cache layer {l}")
    p.check(assert_one_call_equals(p, hidden, [64] * 8, g), o, "one call, overlapped")


def assert_one_call_equals(p, hidden, chunks, want):
    """The benchmark's launch configuration: the prompt in one call, chunks overlapping on four lanes.  Against the
    oracle at the parity bar, and against one call per chunk up to fp32 summation order."""
    import torch
    kv_want = p.kv_gpu()
    p.stage.enable_overlap(4)
    p.kv.reset()
    x = torch.from_numpy(hidden).to(device="cuda:0", dtype=p.td)
    y = to_numpy(p.stage.prefill_chunks(x, chunks, 0, p.kv))
    assert len(p.kv) == sum(chunks)
    # bf16 last-bit differences, compounded over the 8-10 layers of these stages (GPU vs oracle is ~1e-2 here)
    assert rel_l2(y, want) <= 1.2e-2, rel_l2(y, want)
    assert rel_l2(p.kv_gpu(), kv_want) <= 8e-3, rel_l2(p.kv_gpu(), kv_want)
    return y


@pytest.mark.slow
def test_c3_7b_stage_2048_tokens_chunk_sizes_128_to_2048():
    """Config 3: the same stage, 2048-token prompt, chunkings 16x128, 8x256, 4x512, 2x1024 and one shot against
    one oracle run (the oracle's own chunk invariance is pinned on the CPU)."""
    p = Pair(si.LLAMA7B_STAGE, "bf16", seed=30, max_positions=2048, max_chunk_tokens=2048)
    hidden = p.hidden(2048)
    o = []
    for c in range(4):
        o.append(p.oracle.prefill_chunk(hidden[c * 512:(c + 1) * 512], c * 512))
        print(f"oracle chunk {c} done", flush=True)
    o = np.concatenate(o)
    for size in (512, 1024, 2048, 256, 128):
        p.kv.reset()
        g = np.concatenate([p.gpu_chunk(hidden[s:s + size], s) for s in range(0, 2048, size)])
        p.check(g, o, f"chunk size {size}")
        p.check(g[-size:], o[-size:], f"last chunk of size {size}")
        kv = p.kv_gpu()
        for l in range(8):
            p.check(kv[l], p.oracle.kv[l], f"cache layer {l}, chunk size {size}")
        if size == 512:
            g512 = g
    # the launch configuration of the benchmark: the whole prompt in one call, chunks overlapping on the GPU
    import torch
    p.stage.enable_overlap(4)
    x = torch.from_numpy(hidden).to(device="cuda:0", dtype=p.td)
    for chunks in ([512] * 4, [128] * 16):
        p.kv.reset()
        y = to_numpy(p.stage.prefill_chunks(x, chunks, 0, p.kv))
        p.check(y, o, f"one call, chunks {chunks[0]}")
        if chunks[0] == 512:
            assert rel_l2(y, g512) <= 1.2e-2, rel_l2(y, g512)   # fewer K splits: fp32 summation order differs
            kv1 = p.kv_gpu()
            for l in range(8):
                p.check(kv1[l], p.oracle.kv[l], f"cache layer {l}, one call")


@pytest.mark.slow
def test_bf16_long_prefix_8192_cached_positions():
    """One 7B-shaped layer behind a long prompt: the 8192-token prefix goes in as one overlapped call of 2048-token
    chunks; then a 512-token chunk, a ragged short one and a 26-node token tree attend over more than 8192 cached
    positions (several hundred key tiles per query block, rotary angles at large positions)."""
    import torch
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1)
    n_prefix = 8192
    p = Pair(cfg, "bf16", seed=60, max_positions=n_prefix + 640, max_chunk_tokens=2048)
    hidden = p.hidden(n_prefix + 512 + 37 + 1 + 5 + 26)
    o = []
    for s in range(0, n_prefix, 1024):
        o.append(p.oracle.prefill_chunk(hidden[s:s + 1024], s))
        print(f"oracle prefix chunk at {s} done", flush=True)
    p.stage.enable_overlap(4)
    x = torch.from_numpy(hidden[:n_prefix]).to(device="cuda:0", dtype=p.td)
    g = to_numpy(p.stage.prefill_chunks(x, [2048] * 4, 0, p.kv))
    p.check(g, np.concatenate(o), "prefix")
    p.check(g[-2048:], np.concatenate(o)[-2048:], "last prefix chunk")
    pos = n_prefix
    for n in (512, 37, 1, 5):           # the short ones split their 260+ key tiles over 8 workgroups per query block
        h = hidden[pos:pos + n]
        got = p.gpu_chunk(h, pos)
        p.check(got, p.oracle.prefill_chunk(h, pos), f"chunk of {n} at {pos}")
        for rep in range(2):             # the merge order is fixed: same bits whichever workgroup finishes last
            assert np.array_equal(p.gpu_chunk(h, pos), got), (n, rep)
        pos += n
    # a branch forked at the end of the prompt (Sec. V-B): its 5-token chunk reads 8192+ shared positions and its own
    fork = p.kv.fork(pos, pos + 16)
    h = p.hidden(5 + 5, tag=7)
    keep = p.oracle.kv.copy()
    for lo in (0, 5):
        got = p.gpu_chunk(h[lo:lo + 5], pos + lo, kv=fork)
        p.check(got, p.oracle.prefill_chunk(h[lo:lo + 5], pos + lo), f"forked branch, chunk at {pos + lo}")
    assert np.array_equal(p.gpu_chunk(h[5:], pos + 5, kv=fork), got)
    p.check(to_numpy(fork.view())[0][:, :, :10], p.oracle.kv[0, :, :, pos:pos + 10], "fork cache")
    fork.destroy()
    p.oracle.kv[...] = keep
    p.oracle.kv_len = pos
    parents = si.make_token_tree(26, 60)
    h = hidden[pos:pos + 26]
    p.check(p.gpu_tree(h, pos, parents), p.oracle.prefill_tree(h, parents, pos), f"tree at {pos}")
    kv = p.kv_gpu()[0][:, :, :pos + 26]
    for which in range(2):
        p.check(kv[which], p.oracle.kv[0, which, :, :pos + 26], f"cache {'KV'[which]}")


@pytest.mark.slow
def test_bf16_widest_stage_d_model_8192():
    """The widest model the bf16 path accepts (d_model 8192, 64 heads; FFN 28672 as in a 70B-class layer), one
    layer: a 512-token chunk, a 64-token chunk and a 5-token chunk."""
    cfg = dict(si.LLAMA7B_STAGE, d_model=8192, n_heads=64, d_ffn=28672, n_layers=1)
    p = Pair(cfg, "bf16", seed=80, max_positions=640, max_chunk_tokens=512)
    print("weights ready", flush=True)
    chunks = [512, 64, 5]
    hidden = p.hidden(sum(chunks))
    g, o = p.run_both(hidden, chunks)
    row = 0
    for n in chunks:
        p.check(g[row:row + n], o[row:row + n], f"chunk of {n} at {row}")
        row += n
    kv = p.kv_gpu()[0][:, :, :row]
    for which in range(2):
        p.check(kv[which], p.oracle.kv[0, which, :, :row], f"cache {'KV'[which]}")


@pytest.mark.slow
def test_c4_13b_stage_1024_tokens_in_8_chunks_of_128():
    """Config 4: 10 layers of Llama-2-13B shape, bf16, 1024 tokens as 8x128."""
    p = Pair(si.LLAMA13B_STAGE, "bf16", seed=40, max_positions=1024, max_chunk_tokens=128)
    hidden = p.hidden(1024)
    g, o = [], []
    for c in range(8):
        h = hidden[c * 128:(c + 1) * 128]
        g.append(p.gpu_chunk(h, c * 128))
        o.append(p.oracle.prefill_chunk(h, c * 128))
        p.check(g[-1], o[-1], f"chunk {c}")
        print(f"chunk {c} done", flush=True)
    p.check(np.concatenate(g), np.concatenate(o), "hidden_out")
    kv = p.kv_gpu()
    for l in range(10):
        p.check(kv[l], p.oracle.kv[l], f"cache layer {l}")
    p.check(assert_one_call_equals(p, hidden, [128] * 8, np.concatenate(g)), np.concatenate(o), "one call, overlapped")


@pytest.mark.slow
def test_c5_decode_sized_chunks_on_eight_branches_sharing_a_512_token_prefix():
    """Config 5: 8 branches share a 512-token prompt cache, hold 64 private tokens each, and submit a
    5-token chunk (1 token + 4 drafts) with a causal mask inside the chunk."""
    p = Pair(si.LLAMA7B_STAGE, "bf16", seed=50, max_positions=512, max_chunk_tokens=128, oracle_positions=581)
    run_fork_case(p, n_prefix=512, n_private=64, n_chunk=5, n_branches=8)


@pytest.mark.slow
def test_c5_all_eight_branches_in_one_call():
    """Config 5 with the 8 branches batched: 40 rows through the stage at once."""
    p = Pair(si.LLAMA7B_STAGE, "bf16", seed=50, max_positions=512, max_chunk_tokens=128, oracle_positions=581)
    run_batched_branches_case(p, n_prefix=512, n_privates=[64] * 8, n_chunk=5)


@pytest.mark.parametrize("dtype,expanded", [("bf16", False), ("w4", False), ("w4", True)])
def test_random_chunk_lists_rollbacks_and_multi_chunk_calls(dtype, expanded):
    """Seeded random histories of one sequence on a 2-layer 7B-shaped stage: chunks whose lengths sit on and beside
    the tile edges of the kernels (31/32/33 ... 511/512), rollbacks to an earlier position (Sec. V-A) and
    several chunks in one (possibly overlapped) call, every output and the final cache against the oracle."""
    torch = torch_mod()
    sizes_all = [1, 2, 5, 16, 17, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 200, 255, 256, 257, 384, 385, 511, 512]
    rng = np.random.default_rng({"bf16": 11, "w4": 12}[dtype] + int(expanded))
    cap = 1400
    for case in range(2):
        p = Pair(LLAMA7B_2L, dtype, seed=1100 + case, max_positions=cap, max_chunk_tokens=512, w4_expanded=expanded)
        if case == 1:
            p.stage.enable_overlap(int(rng.integers(2, 5)))
        h = p.hidden(cap)
        pos, history = 0, []
        for _ in range(int(rng.integers(4, 8))):
            kind = rng.random()
            if kind < 0.2 and pos > 8:
                pos = int(rng.integers(max(0, pos - 200), pos))
                history.append(f"rollback to {pos}")
            if kind > 0.7 and pos + 700 < cap:
                sizes = [int(rng.choice(sizes_all[:18])) for _ in range(int(rng.integers(2, 5)))]
                x = torch.from_numpy(h[pos:pos + sum(sizes)]).to(device="cuda:0", dtype=p.td)
                y = to_numpy(p.stage.prefill_chunks(x, sizes, pos, p.kv))
                torch.cuda.synchronize()
                want, at = [], pos
                for n in sizes:
                    want.append(p.oracle.prefill_chunk(h[at:at + n], at))
                    at += n
                history.append(f"chunks {sizes} at {pos}")
                p.check(y, np.concatenate(want), "; ".join(history))
                pos = at
            else:
                n = min(int(rng.choice(sizes_all)), cap - pos)
                if n <= 0:
                    break
                history.append(f"{n} at {pos}")
                p.check(p.gpu_chunk(h[pos:pos + n], pos), p.oracle.prefill_chunk(h[pos:pos + n], pos), "; ".join(history))
                pos += n
        assert len(p.kv) == pos
        kv = p.kv_gpu()[:, :, :, :pos]
        for l in range(2):
            p.check(kv[l], p.oracle.kv[l, :, :, :pos], f"cache layer {l} after " + "; ".join(history))


# ------------------------------------------------------------------------------------------------
# 4-bit stage (JUP_BF16_W4; the paper evaluates INT4 models, Sec. VI-A): the GPU reads codes and scales, the
# oracle runs on the matrices they expand to.  Same bar as bf16: codes and scales are exact inputs on both sides.
# ------------------------------------------------------------------------------------------------
def test_w4_two_layer_7b_shape_decode_sized_chunks_tree_and_keep():
    p = Pair(LLAMA7B_2L, "w4", seed=90, max_positions=300, max_chunk_tokens=128)
    hidden = p.hidden(152)
    # up to 16 rows: one row group; 32: two; 40 and 64: four (one pass over the codes each)
    g, o = p.run_both(hidden, [16, 5, 1, 16, 7, 32, 40, 3, 32])
    p.check(g, o, "chunk by chunk")
    row = 0
    for n in [16, 5, 1, 16, 7, 32, 40, 3, 32]:
        p.check(g[row:row + n], o[row:row + n], f"chunk of {n} at {row}")
        row += n
    kv = p.kv_gpu()[:, :, :, :row]
    for l in range(2):
        p.check(kv[l], p.oracle.kv[l, :, :, :row], f"cache layer {l}")
    run_tree_case(p, n_prefix=100, n_tree=64, seed=31)
    run_tree_case(p, n_prefix=37, n_tree=12, seed=32)


def test_w4_smallest_and_odd_widths():
    for d_model, n_heads, d_ffn in ((256, 2, 128), (768, 6, 896)):
        cfg = dict(si.LLAMA7B_STAGE, n_layers=2, d_model=d_model, n_heads=n_heads, d_ffn=d_ffn)
        p = Pair(cfg, "w4", seed=91 + n_heads, max_positions=128, max_chunk_tokens=32)
        hidden = p.hidden(62)
        g, o = p.run_both(hidden, [16, 5, 32, 9])
        p.check(g, o, f"d_model {d_model}")
        run_tree_case(p, n_prefix=20, n_tree=26, seed=33)


def test_w4_batched_branches_equal_one_call_per_branch_bitwise():
    p = Pair(LLAMA7B_2L, "w4", seed=92, max_positions=70, max_chunk_tokens=64, oracle_positions=96)
    run_batched_branches_case(p, n_prefix=70, n_privates=[9, 0, 17, 4, 11, 2, 8, 13], n_chunk=5)   # 40 rows
    run_batched_branches_case(p, n_prefix=33, n_privates=[3, 12, 6], n_chunk=7)                   # 21 rows


def test_w4_overlapped_chunks_equal_one_call_per_chunk_bitwise():
    """The 4-bit projections take the same tiles and splits whether or not chunks overlap: bit-identical results."""
    p = Pair(LLAMA7B_2L, "w4", seed=93, max_positions=200, max_chunk_tokens=64)
    p.stage.enable_overlap(4)
    run_chunks_case(p, [16, 5, 64, 0, 33, 16, 1], pos0_chunks=(16, 9), exact=True)
    y, h = run_chunks_case(p, [16, 16, 16, 16], exact=True)
    p.oracle.reset()
    o = np.concatenate([p.oracle.prefill_chunk(h[i:i + 16], i) for i in range(0, 64, 16)])
    p.check(y, o, "overlapped call")


def test_w4_same_call_twice_is_bitwise_identical_and_zero_codes_give_zero():
    torch = torch_mod()
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1, d_model=512, n_heads=4, d_ffn=640)
    layers = si.make_w4_layers(cfg, seed=95)
    for name in ("wo", "w_down"):           # code 8 everywhere: both projections back to d_model are zero
        layers[0][name][:] = 0x88
    p = Pair(cfg, "w4", seed=95, max_positions=64, max_chunk_tokens=16, layers_np=layers)
    h = p.hidden(13)
    y1 = p.gpu_chunk(h, 0)
    bits1 = kv_bits(p.kv)
    # zero up to fp32 rounding: the offset of the codes leaves as 136 * rowsum(A), summed in another order
    assert np.max(np.abs(y1 - h)) <= 1e-4, "zero output projections must pass the input through"
    p.kv.reset()
    assert np.array_equal(y1, p.gpu_chunk(h, 0))
    assert np.array_equal(bits1, kv_bits(p.kv))
    # the cache of a 4-bit stage holds bf16 entries: one made for the bf16 dtype serves as well
    kvb = jb.KvCache(cfg, "bf16", 64)
    assert np.array_equal(y1, p.gpu_chunk(h, 0, kv=kvb))
    assert np.array_equal(bits1, kv_bits(kvb))


def test_w4_stage_equals_the_bf16_stage_on_weights_both_can_hold():
    """Scales that are powers of two make every expanded weight a bf16 number: the bf16 stage on the expanded
    matrices and the 4-bit stage on the codes then compute the same products and differ by fp32 summation order
    only (two independent GPU paths, same answer; both against the oracle as well)."""
    from oracle import w4
    cfg = LLAMA7B_2L
    layers = si.make_w4_layers(cfg, seed=97)
    rng = np.random.default_rng(97)
    for w in layers:
        for n in w4.MATRIX_NAMES:
            w[n + "_scale"] = np.exp2(rng.integers(-9, -6, size=w[n + "_scale"].shape)).astype(np.float32)
    full = w4.dequantize_layers(layers)
    for w in full:
        for n in w4.MATRIX_NAMES:
            assert np.array_equal(si.round_to_bf16(w[n]), w[n]), n   # exactly representable
    pq = Pair(cfg, "w4", seed=97, max_positions=80, max_chunk_tokens=16, layers_np=layers)
    pb = Pair(cfg, "bf16", seed=97, max_positions=80, max_chunk_tokens=16, layers_np=full)
    h = pq.hidden(53)
    chunks = [16, 16, 5, 16]
    gq, o = pq.run_both(h, chunks)
    gb, _ = pb.run_both(h, chunks)
    pq.check(gq, o, "4-bit stage")
    assert rel_l2(gq, gb) <= 3e-3, rel_l2(gq, gb)
    assert rel_l2(pq.kv_gpu()[:, :, :, :53], pb.kv_gpu()[:, :, :, :53]) <= 3e-3


def test_w4_expanded_stage_runs_long_chunks_on_its_bf16_copy():
    """A 4-bit stage created with w4_expanded: chunks of more than 64 rows take the bf16 projections on
    bf16(scale * (code - 8)), shorter ones stream the codes; both against the oracle on the exact expansion (one
    more rounding of the weights than the codes carry: same bar), cache included."""
    p = Pair(LLAMA7B_2L, "w4", seed=98, max_positions=700, max_chunk_tokens=256, w4_expanded=True)
    chunks = [200, 5, 65, 64, 256, 1, 97]
    h = p.hidden(sum(chunks))
    g, o = p.run_both(h, chunks)
    p.check(g, o, "expanded stage, chunk by chunk")
    row = 0
    for n in chunks:
        p.check(g[row:row + n], o[row:row + n], f"expanded stage, chunk of {n} at {row}")
        row += n
    kv = p.kv_gpu()[:, :, :, :row]
    for l in range(2):
        p.check(kv[l], p.oracle.kv[l, :, :, :row], f"expanded stage, cache layer {l}")
    # up to 64 rows the expanded stage IS the codes-only stage: bit-identical
    lean = Pair(LLAMA7B_2L, "w4", seed=98, max_positions=128, max_chunk_tokens=64, layers_np=p.layers_np)
    p.kv.reset()
    row = 0
    for n in [64, 5, 33]:
        assert np.array_equal(p.gpu_chunk(h[row:row + n], row), lean.gpu_chunk(h[row:row + n], row)), n
        row += n
    assert np.array_equal(kv_bits(p.kv)[..., :row, :], kv_bits(lean.kv)[..., :row, :])


def test_w4_expanded_stage_batched_branches_of_more_than_64_rows():
    """Six branches of 16 tokens in one call are 96 rows: on a stage with the bf16 copy they take the bf16 projections
    (with the per-branch cache append of the QKV epilogue), a single branch's 16 rows the 4-bit ones.  The two read
    different forms of the weights (rounded to bf16 / exact), so they agree with each other only as closely as each
    agrees with the oracle; every branch is checked against the oracle at the usual bar."""
    p = Pair(LLAMA7B_2L, "w4", seed=94, max_positions=70, max_chunk_tokens=128, oracle_positions=110, w4_expanded=True)
    run_batched_branches_case(p, n_prefix=70, n_privates=[9, 0, 17, 4, 11, 2], n_chunk=16, exact=False, close=1.5e-2)


def test_w4_expanded_copy_is_the_rounded_expansion_bitwise():
    """Pins the expansion kernel: a bf16 stage built from round_to_bf16(scale * (code - 8)), computed on the host,
    gives bit-identical results to the expanded 4-bit stage on chunks of more than 64 rows (same kernels, same
    operands), also through the overlapped multi-chunk call."""
    from oracle import w4
    cfg = LLAMA7B_2L
    layers = si.make_w4_layers(cfg, seed=99)
    full = w4.dequantize_layers(layers)
    for w in full:
        for n in w4.MATRIX_NAMES:
            w[n] = si.round_to_bf16(w[n].astype(np.float32))
    pq = Pair(cfg, "w4", seed=99, max_positions=600, max_chunk_tokens=256, layers_np=layers, w4_expanded=True)
    pb = Pair(cfg, "bf16", seed=99, max_positions=600, max_chunk_tokens=256, layers_np=full)
    h = pq.hidden(96 + 256 + 130)
    row = 0
    for n in [96, 256, 130]:
        assert np.array_equal(pq.gpu_chunk(h[row:row + n], row), pb.gpu_chunk(h[row:row + n], row)), n
        row += n
    assert np.array_equal(kv_bits(pq.kv)[..., :row, :], kv_bits(pb.kv)[..., :row, :])
    pq.stage.enable_overlap(4)
    pb.stage.enable_overlap(4)
    yq, _ = run_chunks_case(pq, [128, 128, 128, 98], exact=False)
    yb, _ = run_chunks_case(pb, [128, 128, 128, 98], exact=False)
    assert np.array_equal(yq, yb)


def test_w4_stage_creation_rejects_missing_scales():
    torch = torch_mod()
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1, d_model=256, n_heads=2, d_ffn=128)
    dev = jb.upload_w4_layers(si.make_w4_layers(cfg, seed=96))
    stage = jb.Stage(cfg, "w4", dev, 16)     # complete layers: accepted
    del stage
    ccfg = jb.make_config(cfg, "w4")
    import ctypes
    L = jb.lib()
    arr = (jb.LayerWeights * 1)()
    for n in jb.WEIGHT_NAMES:
        setattr(arr[0], n, dev[0][n].data_ptr())
    for n, field in zip(jb.MATRIX_NAMES, jb.SCALE_FIELDS):
        if field != "s_up":
            setattr(arr[0], field, dev[0][n + "_scale"].data_ptr())
    pb = L.jup_stage_packed_bytes(ctypes.byref(ccfg))
    wb = L.jup_stage_workspace_bytes(ctypes.byref(ccfg), 16)
    packed = torch.empty(pb, dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda:0")
    handle = ctypes.c_void_p()
    rc = L.jup_stage_create(ctypes.byref(ccfg), arr, ctypes.c_void_p(packed.data_ptr()), pb,
                            ctypes.c_void_p(ws.data_ptr()), wb, 16, None, ctypes.byref(handle))
    assert rc == jb.JUP_EINVAL and "scale" in jb.last_error()
