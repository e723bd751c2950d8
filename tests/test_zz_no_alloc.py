"""jup_stage_prefill_chunk_static: the hot path on the library's static scratch, for callers that cannot allocate.
Its output is compared with jup_stage_prefill_chunk's (same kernels: bit for bit, which is inside the parity bar) on
two calls in a row, the second with a smaller input, and with the oracle."""
import numpy as np
import pytest

from helpers import Pair, to_numpy
from paper_2504_08242_amd import binding as jb
from paper_2504_08242_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def bits(t):
    import torch
    return t.view(torch.int32 if t.dtype == torch.float32 else torch.int16).cpu().numpy().copy()


@pytest.mark.parametrize("dtype,cfg,first,second", [
    ("bf16", dict(si.LLAMA7B_STAGE, n_layers=2), 48, 5),
    ("f32", si.TINY, 40, 7),
    ("w4", dict(si.LLAMA7B_STAGE, n_layers=2), 16, 3),
])
def test_static_scratch_call_equals_the_ordinary_call_twice_in_a_row(dtype, cfg, first, second):
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    p = Pair(cfg, dtype, seed=120, max_positions=96, max_chunk_tokens=64)
    h = p.hidden(first + second)
    x1 = torch.from_numpy(h[:first]).to("cuda:0", p.td)
    x2 = torch.from_numpy(h[first:]).to("cuda:0", p.td)
    # the ordinary entry point on the caller's workspace
    want1 = p.stage.prefill_chunk(x1, 0, p.kv)
    want2 = p.stage.prefill_chunk(x2, first, p.kv)
    torch.cuda.synchronize()
    want_kv = bits(p.kv.buf)
    o1 = p.oracle.prefill_chunk(h[:first], 0)
    o2 = p.oracle.prefill_chunk(h[first:], first)
    # the static entry point on a fresh cache; the workspace of the stage is poisoned to show it is not used
    kv2 = jb.KvCache(cfg, dtype, 96)
    p.stage.workspace.fill_(0xFF)
    y1, y2 = torch.empty_like(x1), torch.empty_like(x2)
    p.stage.prefill_chunk_static(x1, 0, kv2, y1)
    p.stage.prefill_chunk_static(x2, first, kv2, y2)          # smaller input, right behind the first call
    torch.cuda.synchronize()
    assert len(kv2) == first + second
    assert np.array_equal(bits(y1), bits(want1)) and np.array_equal(bits(y2), bits(want2))
    assert np.array_equal(bits(kv2.buf), want_kv)
    assert (p.stage.workspace == 0xFF).all(), "the static call wrote into the stage's workspace"
    p.check(to_numpy(y1), o1, "first call vs oracle")
    p.check(to_numpy(y2), o2, "second call vs oracle")
    # ... and again after the smaller call, from the start: nothing in the scratch has to survive or start at zero
    kv2.reset()
    p.stage.prefill_chunk_static(x1, 0, kv2, y1)
    torch.cuda.synchronize()
    assert np.array_equal(bits(y1), bits(want1))


def test_static_scratch_call_behind_a_long_cache_equals_the_ordinary_call():
    """Key-split attention keeps partial results and arrival counters in the scratch: the static array must serve them
    as the workspace does, on two calls in a row (the second smaller)."""
    import torch
    cfg = dict(si.LLAMA7B_STAGE, n_layers=2)
    p = Pair(cfg, "bf16", seed=122, max_positions=1200, max_chunk_tokens=300)
    h = p.hidden(1100 + 48 + 5)
    x = torch.from_numpy(h).to("cuda:0", p.td)
    for c in range(4):
        p.stage.prefill_chunk(x[c * 275:(c + 1) * 275], c * 275, p.kv)
    want1 = p.stage.prefill_chunk(x[1100:1148], 1100, p.kv)
    want2 = p.stage.prefill_chunk(x[1148:], 1148, p.kv)
    torch.cuda.synchronize()
    want_kv = bits(p.kv.buf)
    p.kv.truncate(1100)
    y1, y2 = torch.empty_like(want1), torch.empty_like(want2)
    p.stage.prefill_chunk_static(x[1100:1148], 1100, p.kv, y1)
    p.stage.prefill_chunk_static(x[1148:], 1148, p.kv, y2)
    torch.cuda.synchronize()
    assert np.array_equal(bits(y1), bits(want1)) and np.array_equal(bits(y2), bits(want2))
    assert np.array_equal(bits(p.kv.buf), want_kv)


def test_static_scratch_call_rejects_what_does_not_fit_and_validates_like_the_ordinary_call():
    import torch
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1)
    p = Pair(cfg, "bf16", seed=121, max_positions=400, max_chunk_tokens=16)
    x = torch.zeros((224, cfg["d_model"]), device="cuda:0", dtype=torch.bfloat16)
    y = torch.empty_like(x)
    with pytest.raises(jb.JupiterError) as e:                 # 224 tokens of a 7B-shaped stage need more than 48 MiB
        p.stage.prefill_chunk_static(x, 0, p.kv, y)
    assert e.value.status == jb.JUP_ECAP and "static" in str(e.value) and len(p.kv) == 0
    p.stage.prefill_chunk_static(x[:192], 0, p.kv, y[:192])   # the largest that fits; above the stage's max_chunk_tokens
    assert len(p.kv) == 192
    with pytest.raises(jb.JupiterError) as e:                 # a hole
        p.stage.prefill_chunk_static(x[:4], 200, p.kv, y[:4])
    assert e.value.status == jb.JUP_EPOS and len(p.kv) == 192
    p.stage.prefill_chunk_static(x[:0], 192, p.kv, y[:0])     # empty chunk: no-op
    torch.cuda.synchronize()
    assert len(p.kv) == 192
