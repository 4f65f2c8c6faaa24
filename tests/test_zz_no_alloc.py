"""saw_paged_decode_attn_static (the entry point that allocates nothing: split-KV partial results in a
library-held static device array) against saw_paged_decode_attn with a caller-provided workspace: same
kernels, so the outputs must be bit-identical, on two calls in a row, the second with a smaller input
(what the first call left in the shared array must not matter)."""
import ctypes

import numpy as np
import pytest
import torch

import gpu_cases as gc
import parity
from oracle import saw_oracle as O
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def _run_both(saw, w, num_splits):
    ref = gc.oracle_fill(w)
    cache = gc.upload_cache(ref, w, saw)
    pt = torch.from_numpy(w.page_table).cuda()
    sl = torch.from_numpy(w.seq_lens).cuda()
    q = synth.gen_q(w).cuda()
    bound = int(w.seq_lens.max())
    splits, _ = saw.decode_plan(cache, w.batch, bound, num_splits)
    want = saw.paged_decode_attn(cache, q, pt, sl, max_seq_len=bound, num_splits=num_splits)
    out = torch.full_like(want, float("nan"))
    saw.paged_decode_attn_static(cache, q, pt, sl, out, max_seq_len=bound, num_splits=num_splits)
    torch.cuda.synchronize()
    assert torch.equal(out, want), f"{w.name}: static-scratch call differs from the workspace call"
    o_ref = O.paged_decode_attn(ref, q.float().cpu().numpy(), w.page_table, w.seq_lens, w.had_block, w.rotate_mask)
    err = parity.attn_error(out.cpu().numpy(), o_ref)
    print(f"[{w.name} B={w.batch} splits={splits}] err vs oracle={err:.2e}", flush=True)
    assert err < 2e-3
    return splits


def test_static_scratch_matches_workspace_call_twice_second_smaller(saw):
    # first call: several partitions per sequence, so the scratch holds partial results
    s1 = _run_both(saw, synth.make_workload("llama8b", batch=5, ctx=(2600, 4000)), num_splits=0)
    assert s1 > 1
    # second call, smaller in every dimension, partitions again: stale records of the first call lie around it
    s2 = _run_both(saw, synth.make_workload("tiny", batch=2, ctx=(70, 200)), num_splits=3)
    assert s2 > 1
    # and a call without partitions (the scratch is passed but unused)
    _run_both(saw, synth.make_workload("tiny", batch=3, ctx=(1, 90)), num_splits=1)


def test_static_scratch_rejects_calls_beyond_its_size(saw):
    cache = saw.Cache(8, 8, 128, 128)
    B, Hq = 64, 64
    q = torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device="cuda")
    pt = torch.zeros((B, 8192), dtype=torch.int32, device="cuda")
    sl = torch.zeros(B, dtype=torch.int32, device="cuda")
    out = torch.zeros((B, Hq, 128), device="cuda")
    assert saw.decode_workspace_bytes(cache, B, Hq, 131072, 64) > (16 << 20)
    with pytest.raises(saw.SawError) as e:
        saw.paged_decode_attn_static(cache, q, pt, sl, out, max_seq_len=131072, num_splits=64)
    assert e.value.code == -5 and "static scratch" in str(e.value)
