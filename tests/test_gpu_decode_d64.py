"""Parity of the head_dim 64 INT4 decode with the fp64 oracle (Sec. 4.1, App. A.4: the block-diagonal
rotation only needs h | d, so 64-channel heads are served too).

With an even number of kv heads and at most 4 query heads per kv head the matrix-core kernel runs on
pairs of kv heads; other shapes take the vector-ALU kernel.  Every way the kernel hands out work is
driven here at head_dim 64: one partition, split-KV with the merge pass, several wavefronts per
partition, pair mode, longest-first order, and the append entry point (store launch + decode).
"""
import numpy as np
import pytest
import torch

import test_gpu_append as TA
import test_gpu_decode as TD
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def _w(name="highconc", **kw):
    kw.setdefault("head_dim", 64)
    kw.setdefault("had_block", 64)
    return synth.make_workload(name, **kw)


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (8, 2), (8, 8), (32, 8), (6, 6)])
def test_head_pairs_group_sizes(saw, Hq, Hkv):
    TD._decode_case(saw, _w(batch=3, ctx=(20, 150), n_q_heads=Hq, n_kv_heads=Hkv))


@pytest.mark.parametrize("Hq,Hkv", [(3, 3), (6, 3), (16, 2), (5, 5)])
def test_shapes_outside_the_pair_kernel(saw, Hq, Hkv):
    """Odd kv head counts and 8 query heads per kv head: the vector-ALU kernel."""
    TD._decode_case(saw, _w(batch=3, ctx=(20, 150), n_q_heads=Hq, n_kv_heads=Hkv))


@pytest.mark.parametrize("h,mask", [(1, 3), (16, 3), (32, 3), (64, 3), (64, 1), (32, 2), (64, 0)])
@pytest.mark.parametrize("sign_seed", [None, 5])
def test_head_pairs_block_sizes_masks_signs(saw, h, mask, sign_seed):
    w = _w(batch=2, ctx=(40, 200), n_q_heads=16, n_kv_heads=4, had_block=h, rotate_mask=mask, sign_seed=sign_seed)
    TD._decode_case(saw, w)


@pytest.mark.parametrize("splits", [1, 2, 3, 0])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 4), (16, 4)])
def test_head_pairs_split_kv(saw, splits, Hq, Hkv):
    w = _w("tiny", batch=3, ctx=(130, 700), n_q_heads=Hq, n_kv_heads=Hkv)
    TD._decode_case(saw, w, num_splits=splits, end_to_end=False)


def test_head_pairs_ragged_with_empty_and_single(saw):
    w = _w(batch=7, seq_lens=[0, 1, 15, 16, 17, 64, 333], n_q_heads=16, n_kv_heads=4)
    o, _ = TD._decode_case(saw, w, num_splits=2)
    assert not o[0].any()
    o, _ = TD._decode_case(saw, w, num_splits=1, end_to_end=False)
    assert not o[0].any()


@pytest.mark.parametrize("B,Hq,Hkv", [(70, 32, 8), (140, 16, 4), (150, 32, 8), (255, 8, 8), (300, 8, 8), (340, 16, 8),
                                      (340, 32, 8), (600, 8, 8)])
def test_head_pairs_many_sequences(saw, B, Hq, Hkv):
    """More (sequence, head pair) items than compute units: pair mode (blocks of two wavefronts, of four
    from 576 to 1024 items: the third and fourth case; of four over three sequences from 1152 to 1536 items:
    the sixth, while the seventh, with eight query rows per head pair, stays with blocks of two), longest first
    beyond 2048 items (the last case).
    Lengths include empty sequences and many ties."""
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 200, size=B)
    lens[rng.integers(0, B, size=B // 5)] = 64
    lens[:3] = [0, 199, 1]
    w = _w(batch=B, seq_lens=lens, n_q_heads=Hq, n_kv_heads=Hkv)
    TD._decode_case(saw, w, num_splits=1, end_to_end=False)
    TD._decode_case(saw, w, num_splits=0, end_to_end=False)


def test_head_pairs_long_context_several_wavefronts(saw):
    w = _w("longctx1", ctx=9000, n_q_heads=8, n_kv_heads=2)
    TD._decode_case(saw, w, num_splits=0, end_to_end=False)
    TD._decode_case(saw, w, num_splits=1, end_to_end=False)       # one partition, four wavefronts on it
    TD._decode_case(saw, w, num_splits=37, end_to_end=False)


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float16])
def test_head_pairs_output_and_query_dtypes(saw, out_dtype):
    w = _w("tiny", batch=2, ctx=75, n_q_heads=8, n_kv_heads=4)
    TD._decode_case(saw, w, out_dtype=out_dtype, q_dtype=torch.float32, sm_scale=0.11)


def test_head_pairs_fp16_cache_input(saw):
    TD._decode_case(saw, _w("tiny", batch=2, ctx=(30, 300), n_q_heads=8, n_kv_heads=2, dtype=torch.float16))


@pytest.mark.parametrize("B,Hq,Hkv,ctx", [(3, 8, 4, (20, 150)), (70, 32, 8, (1, 120)), (150, 16, 8, (0, 200)),
                                          (2, 8, 2, (700, 900))])
def test_append_then_attend(saw, B, Hq, Hkv, ctx):
    """saw_append_decode_attn at head_dim 64: the store launch, then the decode over one more token."""
    TA._case(saw, _w(batch=B, ctx=ctx, n_q_heads=Hq, n_kv_heads=Hkv))


@pytest.mark.parametrize("h,mask,sign_seed", [(64, 3, 5), (16, 3, None), (32, 1, 6), (64, 2, None), (1, 3, None)])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (16, 4)])
def test_append_block_sizes_masks_signs(saw, h, mask, sign_seed, Hq, Hkv):
    """The decode kernel's own append at head_dim 64: the new token's bytes per kv head of a pair."""
    TA._case(saw, _w(batch=4, ctx=(1, 200), n_q_heads=Hq, n_kv_heads=Hkv, had_block=h, rotate_mask=mask,
                     sign_seed=sign_seed))


def test_append_unmapped_page_and_odd_kv_heads(saw):
    # (the unmapped token must open a page of its own, or cached tokens would lose their page with it)
    TA._case(saw, _w(batch=3, seq_lens=[40, 64, 95], n_q_heads=8, n_kv_heads=4), unmapped=(1,))
    TA._case(saw, _w(batch=3, ctx=(20, 150), n_q_heads=6, n_kv_heads=3))        # store launch + decode
