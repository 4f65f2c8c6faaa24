"""Parity of saw_flatten_dequant (INT4 pages -> dense 16-bit / fp32 K and V, optionally rotated back)
with the oracle's read-back.  Both sides read the same bytes: the cache the oracle's store wrote."""
import numpy as np
import pytest
import torch

import gpu_cases as gc
from oracle import saw_oracle as O
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu

# |got - ref| <= RTOL[dtype] * |ref| + ATOL_REL * max|ref|: half an ulp of the output type on each
# element, plus the fp32 arithmetic's error relative to the largest value of the tensor
RTOL = {torch.float32: 0.0, torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -11}
ATOL_REL = 2e-6


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def _check(got, ref, dtype, what):
    got = got.float().cpu().numpy().astype(np.float64)
    bound = RTOL[dtype] * np.abs(ref) + ATOL_REL * np.abs(ref).max()
    if dtype == torch.float16:
        bound = bound + 2.0 ** -25                                    # fp16 subnormal spacing
    bad = np.abs(got - ref) > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside the bound, worst {np.abs(got - ref).max():.3e}"


def _case(saw, w, unrotate, dtype, ranges=None):
    ref = gc.oracle_fill(w)
    cache = gc.upload_cache(ref, w, saw)
    pt = torch.from_numpy(w.page_table).cuda()
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        for (p0, p1) in (ranges or [(0, L), (5, min(L, 37)), (L - 1, L), (16, min(L, 48))]):
            if p1 <= p0:
                continue
            k, v = saw.flatten_dequant(cache, pt, b, p0, p1, unrotate=unrotate, out_dtype=dtype)
            kr, vr = O.dequant_pages(ref, w.page_table, b, p0, p1, w.had_block, w.rotate_mask, unrotate=unrotate,
                                     signs=w.signs, dense=w.dense)
            tag = f"[{w.name} h={w.had_block} d={w.head_dim} mask={w.rotate_mask} unrot={unrotate} {dtype} seq {b} [{p0},{p1})]"
            _check(k, kr, dtype, tag + " K")
            _check(v, vr, dtype, tag + " V")
    return cache, ref, pt


@pytest.mark.parametrize("h", [1, 16, 32, 64, 128])
@pytest.mark.parametrize("unrotate", [False, True])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_block_sizes_d128(saw, h, unrotate, dtype):
    _case(saw, synth.make_workload("tiny", batch=2, ctx=(20, 90), had_block=h), unrotate, dtype)


@pytest.mark.parametrize("h", [1, 16, 32, 64])
@pytest.mark.parametrize("unrotate", [False, True])
def test_block_sizes_mha_d64(saw, h, unrotate):
    _case(saw, synth.make_workload("prefill_mha", ctx=70, had_block=h), unrotate, torch.float16)


@pytest.mark.parametrize("mask", [0, 1, 2, 3])
def test_rotate_masks(saw, mask):
    _case(saw, synth.make_workload("llama8b", batch=1, ctx=50, rotate_mask=mask), True, torch.bfloat16)


def test_rotated_back_values_are_the_inputs_up_to_the_quantisation_step(saw):
    w = synth.make_workload("tiny", batch=1, ctx=120)
    cache, ref, pt = _case(saw, w, True, torch.float32, ranges=[(0, 120)])
    K, V = synth.gen_kv(w, 0, 0, 120)
    k, v = saw.flatten_dequant(cache, pt, 0, 0, 120, unrotate=True, out_dtype=torch.float32)
    for got, x, m in ((k, K, ref["k_meta"]), (v, V, ref["v_meta"])):
        # an orthonormal rotation keeps the error vector's norm: at most sqrt(d) half-steps
        assert (got.cpu() - x.float()).norm(dim=-1).max() <= 0.51 * m[..., 0].max() * w.head_dim ** 0.5


def test_large_zero_points_cancel_exactly(saw):
    """Vectors far from zero (|z| in the thousands): the zero-point term must not leak into channels
    where it cancels."""
    w = synth.make_workload("tiny", batch=1, ctx=40, scales="outlier4x2000")
    _case(saw, w, True, torch.float32)
    _case(saw, w, False, torch.float32)


def test_single_tensor_strided_output_and_untouched_rows(saw):
    w = synth.make_workload("tiny", batch=2, ctx=60)
    ref = gc.oracle_fill(w)
    cache = gc.upload_cache(ref, w, saw)
    pt = torch.from_numpy(w.page_table).cuda()
    n, Hkv, d = 33, w.n_kv_heads, w.head_dim
    wide = torch.full((n, Hkv * d + 64), 7.0, dtype=torch.bfloat16, device="cuda")
    k_view = wide[:, :Hkv * d].view(n, Hkv, d)                          # token stride Hkv*d + 64
    k, v = saw.flatten_dequant(cache, pt, 1, 9, 9 + n, unrotate=True, want_v=False, k_out=k_view)
    assert v is None
    kr, _ = O.dequant_pages(ref, w.page_table, 1, 9, 9 + n, w.had_block, w.rotate_mask, unrotate=True)
    _check(k_view, kr, torch.bfloat16, "strided K")
    assert (wide[:, Hkv * d:] == 7.0).all()                             # the gap between tokens is not written
    k2, v2 = saw.flatten_dequant(cache, pt, 1, 9, 9, unrotate=True)     # empty range: no-op
    assert k2.numel() == 0 and v2.numel() == 0


@pytest.mark.parametrize("name,dtype", [("prefill", torch.bfloat16), ("prefill_mha", torch.float16)])
def test_full_size_prefill_range(saw, name, dtype):
    """32768 tokens, every element compared (the size the benchmark times)."""
    w = synth.make_workload(name)
    _case(saw, w, True, dtype, ranges=[(0, 32768)])


@pytest.mark.parametrize("Hkv", [1, 2, 3, 6])
@pytest.mark.parametrize("h,mask", [(64, 3), (16, 1), (32, 2), (1, 3)])
def test_d64_head_pairs_and_odd_head_counts(saw, Hkv, h, mask):
    """head_dim 64: an even head count takes the two-heads-per-wavefront path, an odd one the one-head path."""
    w = synth.make_workload("prefill_mha", batch=2, seq_lens=[83, 16], n_kv_heads=Hkv, n_q_heads=Hkv,
                            had_block=h, rotate_mask=mask, sign_seed=3 if h == 32 else None)
    _case(saw, w, True, torch.bfloat16)
    _case(saw, w, True, torch.float32, ranges=[(3, 70)])
    _case(saw, w, False, torch.float16)
