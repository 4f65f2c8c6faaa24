"""Randomised Hadamard (a +/-1 diagonal in front of the block Hadamard, Sec. 3) through every entry
point of the HIP path, against the oracle's R = diag(sigma) H_blk on the same seeded inputs.  The
drivers are the ones of the other GPU test files; the workloads carry a random sign vector."""
import numpy as np
import pytest
import torch

import test_gpu_append as TA
import test_gpu_decode as TD
import test_gpu_flatten as TF
import test_gpu_store as TS
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def test_cache_descriptor_carries_the_bits(saw):
    sg = synth.random_signs(128, 3)
    c = saw.Cache(2, 1, 128, 64, signs=sg)
    bits = c.struct().sign_bits
    for ch in range(128):
        assert ((bits[ch // 32] >> (ch % 32)) & 1) == (1 if sg[ch] < 0 else 0)
    # bits beyond head_dim are refused
    bad = saw.Cache(2, 1, 64, 16, device="cuda")
    bad.sign_bits[3] = 1
    K = torch.zeros((1, 1, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(saw.SawError):
        saw.rotate_quant_store(bad, K, K, torch.zeros((1, 1), dtype=torch.int32, device="cuda"),
                               torch.zeros((1, 2), dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("h", [16, 32, 64, 128])
@pytest.mark.parametrize("mask", [3, 1, 2])
def test_store_codes_with_signs(saw, h, mask):
    w = synth.make_workload("prefill", ctx=300, had_block=h, rotate_mask=mask, sign_seed=10 * h + mask)
    assert (w.signs < 0).any() and (w.signs > 0).any()
    TS._run(saw, w)


def test_store_codes_with_signs_mha_and_fp16(saw):
    TS._run(saw, synth.make_workload("prefill_mha", ctx=200, had_block=32, sign_seed=4))
    TS._run(saw, synth.make_workload("prefill", ctx=130, had_block=64, dtype=torch.float16, sign_seed=5))


def test_signs_change_the_codes_and_plain_cache_ignores_them(saw):
    """With h = 1 (no rotation) the sign bits have no effect; with rotation they change the bytes."""
    w0 = synth.make_workload("tiny", batch=1, ctx=64, had_block=1)
    w1 = synth.make_workload("tiny", batch=1, ctx=64, had_block=1, sign_seed=8)
    a = TS._run(saw, w0)[2]
    b = TS._run(saw, w1)[2]
    assert np.array_equal(a["k_codes"], b["k_codes"]) and np.array_equal(a["v_meta"], b["v_meta"])
    c = TS._run(saw, synth.make_workload("tiny", batch=1, ctx=64, had_block=128))[2]
    d = TS._run(saw, synth.make_workload("tiny", batch=1, ctx=64, had_block=128, sign_seed=8))[2]
    assert not np.array_equal(c["k_codes"], d["k_codes"])


@pytest.mark.parametrize("name,kw", [("tiny", dict(batch=3, ctx=(40, 300))),                       # G = 4, one partition
                                     ("tiny", dict(batch=2, ctx=(200, 900), rotate_mask=1)),      # K only
                                     ("tiny", dict(batch=2, ctx=(200, 900), rotate_mask=2)),      # V only
                                     ("longctx1", dict(ctx=3000, had_block=64)),                  # G = 8, split-KV + merge
                                     ("highconc", dict(batch=70, ctx=(1, 200))),                  # pair mode
                                     ("prefill_mha", dict(ctx=150, had_block=16))])               # d = 64 path
def test_decode_with_signs(saw, name, kw):
    w = synth.make_workload(name, sign_seed=21, **kw)
    TD._decode_case(saw, w)


@pytest.mark.parametrize("splits", [1, 3])
def test_decode_with_signs_forced_splits(saw, splits):
    w = synth.make_workload("tiny", batch=3, ctx=(130, 700), had_block=32, sign_seed=22)
    TD._decode_case(saw, w, num_splits=splits, end_to_end=False)


@pytest.mark.parametrize("name,kw", [("tiny", dict(batch=3, ctx=(40, 300))),
                                     ("highconc", dict(batch=70, ctx=(1, 200))),
                                     ("tiny", dict(batch=2, ctx=(100, 400), rotate_mask=1)),
                                     ("prefill_mha", dict(ctx=100, had_block=16))])                # unfused fallback (d = 64)
def test_fused_append_with_signs(saw, name, kw):
    TA._case(saw, synth.make_workload(name, sign_seed=23, **kw))


@pytest.mark.parametrize("h,mask", [(16, 3), (64, 3), (128, 3), (128, 1), (32, 2)])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_flatten_with_signs(saw, h, mask, dtype):
    w = synth.make_workload("tiny", batch=2, ctx=(20, 90), had_block=h, rotate_mask=mask, sign_seed=24 + h)
    TF._case(saw, w, True, dtype)
    TF._case(saw, w, False, dtype)


def test_flatten_with_signs_d64(saw):
    w = synth.make_workload("prefill_mha", ctx=70, had_block=32, sign_seed=9)
    TF._case(saw, w, True, torch.float16)


@pytest.mark.parametrize("unrotate", [False, True])
def test_dequant_pages_with_signs(saw, unrotate):
    for name, kw in (("tiny", dict(batch=2, ctx=90)), ("prefill_mha", dict(ctx=70, had_block=16)),
                     ("llama8b", dict(batch=1, ctx=50, rotate_mask=1))):
        TS.test_dequant_pages(saw, name, dict(kw, sign_seed=31), unrotate)
