"""Parity of the learned per-layer rotation (App. A.3: q^ = (q H_b) R_l, k^ = (k H_b) R_l, the same for V)
through every call that supports it, against the oracle, with a seeded random orthogonal matrix standing in
for a calibrated R_l (the calibration needs model queries that are not available here)."""
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


def test_prepared_buffer_holds_the_matrix_its_transpose_and_three_limbs(saw):
    """The fp32 planes are copies; hi + mid + lo of the bf16 limb planes, read back through the documented
    operand order, reproduce every entry to 2^-24 of its magnitude (plus a bf16 subnormal floor)."""
    d = 128
    R = synth.random_orthogonal(d, 3)
    buf = saw.prepare_dense_rotation(R, d)
    torch.cuda.synchronize()
    raw = buf.cpu().numpy()
    f = raw[:2 * d * d * 4].view(np.float32).reshape(2, d, d)
    assert np.array_equal(f[0], R.astype(np.float32)) and np.array_equal(f[1], R.T.astype(np.float32))
    limbs = raw[2 * d * d * 4:].view(np.uint16).reshape(3, 8, 4, 64, 8).astype(np.uint32)
    vals = (limbs << 16).view(np.float32).astype(np.float64).sum(axis=0)          # [J][a][lane][e]
    for J in range(8):
        for a in range(4):
            for lane in range(64):
                m, rg = lane % 16, lane // 16
                j = 32 * (J // 2) + 8 * (m // 4) + 4 * (J % 2) + (m % 4)
                i0 = 32 * a + 8 * rg
                want = R[i0:i0 + 8, j]
                assert np.all(np.abs(vals[J, a, lane] - want) <= np.abs(want) * 2.0 ** -23 + 1e-30)


@pytest.mark.parametrize("name,kw", [
    ("tiny", dict()),                                              # fp16, h = 128, K and V
    ("llama8b", dict(batch=2, ctx=(40, 300))),                     # bf16
    ("highconc", dict(batch=3, ctx=(20, 150), had_block=16)),
    ("highconc", dict(batch=2, ctx=70, had_block=1)),              # the learned rotation alone
    ("tiny", dict(batch=2, ctx=90, rotate_mask=1)),                # K only: V stored without any rotation
    ("tiny", dict(batch=2, ctx=90, rotate_mask=2, had_block=32)),
    ("tiny", dict(batch=2, ctx=90, sign_seed=4, had_block=64)),    # diag(sigma) H_b R_l
])
def test_store_with_learned_rotation(saw, name, kw):
    w = synth.make_workload(name, dense_seed=17, **kw)
    cache, ref, recs, _ = gc.fill_caches(w, saw, order_rng=np.random.default_rng(1))
    res = gc.compare_store(gc.cache_to_numpy(cache, w), ref, recs)
    print(f"[{name} {kw}] {res}", flush=True)
    parity.assert_store_ok(res)
    assert res["untouched_ok"]


@pytest.mark.parametrize("kw,splits", [
    (dict(batch=3, ctx=(130, 700)), 0), (dict(batch=3, ctx=(130, 700)), 3), (dict(batch=3, ctx=(130, 700)), 1),
    (dict(batch=2, ctx=(40, 200), rotate_mask=1), 0), (dict(batch=2, ctx=(40, 200), rotate_mask=2), 2),
    (dict(batch=2, ctx=(40, 200), had_block=1), 0), (dict(batch=2, ctx=100, sign_seed=9, had_block=32), 0),
    (dict(batch=2, ctx=(40, 200), n_q_heads=64), 0), (dict(batch=2, ctx=(40, 200), n_q_heads=8), 2),
])
def test_decode_with_learned_rotation(saw, kw, splits):
    import test_gpu_decode as TD
    w = synth.make_workload("tiny", dense_seed=23, **kw)
    TD._decode_case(saw, w, num_splits=splits)


@pytest.mark.parametrize("B,Hkv", [(70, 8), (150, 8), (200, 8)])
def test_decode_with_learned_rotation_pair_mode(saw, B, Hkv):
    import test_gpu_decode as TD
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 200, size=B)
    lens[:3] = [0, 199, 1]
    w = synth.make_workload("highconc", batch=B, seq_lens=lens, n_q_heads=4 * Hkv, n_kv_heads=Hkv, dense_seed=5)
    TD._decode_case(saw, w, end_to_end=False)


@pytest.mark.parametrize("kw", [dict(batch=3, seq_lens=[0, 47, 200]), dict(batch=3, seq_lens=[5, 64, 130], rotate_mask=1),
                                dict(batch=2, ctx=2000), dict(batch=3, seq_lens=[0, 47, 200], had_block=1),
                                dict(batch=2, seq_lens=[33, 90], n_q_heads=64)])
def test_append_with_learned_rotation(saw, kw):
    import test_gpu_append as TA
    TA._case(saw, synth.make_workload("llama8b", dense_seed=29, **kw))


def test_append_with_learned_rotation_pair_mode(saw):
    import test_gpu_append as TA
    rng = np.random.default_rng(12)
    lens = rng.integers(0, 200, size=150)
    TA._case(saw, synth.make_workload("highconc", batch=150, seq_lens=lens, dense_seed=31))


@pytest.mark.parametrize("mask,h", [(3, 128), (1, 64), (2, 16), (3, 1)])
@pytest.mark.parametrize("unrotate", [False, True])
def test_dequant_pages_with_learned_rotation(saw, mask, h, unrotate):
    w = synth.make_workload("tiny", batch=2, ctx=90, rotate_mask=mask, had_block=h, dense_seed=41)
    ref = gc.oracle_fill(w)
    cache = gc.upload_cache(ref, w, saw)
    pt = torch.from_numpy(w.page_table).cuda()
    for b in range(w.batch):
        for (p0, p1) in [(0, 90), (5, 37), (89, 90)]:
            k, v = saw.dequant_pages(cache, pt, b, p0, p1, unrotate=unrotate)
            kr, vr = O.dequant_pages(ref, w.page_table, b, p0, p1, h, mask, unrotate=unrotate, dense=w.dense)
            for a, r in ((k, kr), (v, vr)):
                assert np.abs(a.cpu().numpy().astype(np.float64) - r).max() <= 4e-6 * np.abs(r).max()
    if unrotate:                                                   # back in the input space, up to the quantisation step
        K, _ = synth.gen_kv(w, 0, 0, 90)
        k, _ = saw.dequant_pages(cache, pt, 0, 0, 90, unrotate=True)
        s = ref["k_meta"][..., 0].max()
        assert (k.cpu() - K.float()).abs().max() <= 0.51 * s * (w.head_dim ** 0.5)


def test_flatten_with_learned_rotation_as_stored_only(saw):
    import test_gpu_flatten as TF
    w = synth.make_workload("tiny", batch=1, ctx=80, dense_seed=43)
    TF._case(saw, w, False, torch.bfloat16)
    cache = gc.upload_cache(gc.oracle_fill(w), w, saw)
    with pytest.raises(saw.SawError) as e:
        saw.flatten_dequant(cache, torch.from_numpy(w.page_table).cuda(), 0, 0, 80, unrotate=True)
    assert e.value.code == -1


def test_learned_rotation_needs_head_dim_128(saw):
    assert saw.lib().saw_dense_rotation_bytes(64) == 0 and saw.lib().saw_dense_rotation_bytes(128) == 224 * 1024
    w = synth.make_workload("highconc", batch=2, ctx=40, head_dim=64, had_block=64, n_q_heads=8, n_kv_heads=4)
    cache = saw.Cache(w.num_pages, w.n_kv_heads, 64, 64)
    cache.dense_rot = torch.zeros(1024, dtype=torch.uint8, device="cuda")          # any non-null pointer
    K, V = synth.gen_kv(w, 0, 0, 40, device="cuda")
    with pytest.raises(saw.SawError) as e:
        saw.rotate_quant_store(cache, K, V, torch.from_numpy(w.page_table).cuda(),
                               torch.from_numpy(synth.slots_for(0, 0, 40)).cuda())
    assert e.value.code == -1
