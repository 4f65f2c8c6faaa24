"""The entry points enqueue kernels only (no allocation, no memset, no synchronisation), so a caller
can capture them into a HIP graph.  Every replay is checked against the eager result, with the
program's own eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import gpu_cases as gc
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name,kw", [("highconc", dict(batch=70, ctx=(1, 200))),      # 560 items: one launch, ...
                                     ("highconc", dict(batch=80, ctx=(1, 200))),      # ... 640: pair blocks of four
                                     ("highconc", dict(batch=200, ctx=(1, 120))),     # ... 1600: pair blocks of two
                                     ("highconc", dict(batch=150, ctx=(1, 150), head_dim=64, had_block=64)),  # head pairs
                                     ("tiny", dict(batch=3, ctx=(130, 700))),          # small batch: blocks of eight wavefronts, one launch
                                     ("tiny", dict(batch=3, ctx=(2600, 3000)))])       # split-KV + merge kernel
def test_decode_step_replays_from_a_graph(saw, name, kw):
    w = synth.make_workload(name, **kw)
    cache, _, _, pt = gc.fill_caches(w, saw, with_ref=False)
    B = w.batch
    lens = torch.from_numpy(w.seq_lens).cuda()
    max_len = int(w.seq_lens.max())
    Kn = torch.cat([synth.gen_kv(w, b, int(w.seq_lens[b]), int(w.seq_lens[b]) + 1)[0] for b in range(B)]).cuda()
    Vn = torch.cat([synth.gen_kv(w, b, int(w.seq_lens[b]), int(w.seq_lens[b]) + 1)[1] for b in range(B)]).cuda()
    q = synth.gen_q(w).cuda()
    out = torch.empty((B, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(saw.decode_workspace_bytes(cache, B, w.n_q_heads, max_len + 1), dtype=torch.uint8, device="cuda")

    def step():
        saw.append_decode_attn(cache, Kn, Vn, q, pt, lens, max_seq_len=max_len, out=out, workspace=ws)

    step()
    torch.cuda.synchronize()
    ref = out.clone()
    ref_codes = cache.k_codes.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        out.fill_(float("nan"))                      # eager work between replays
        scratch = (q.float() * (rep + 1)).sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"replay {rep} differs from the eager result"
        assert torch.equal(cache.k_codes, ref_codes)
        assert np.isfinite(float(scratch))
