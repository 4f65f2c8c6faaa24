"""The C-ABI library loads without a GPU, exports every symbol the header declares, and rejects
bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_19157_amd import build
        build.build_library()
    return binding


def _declared():
    src = open(os.path.join(ROOT, "include", "saw.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(saw_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(saw):
    names = _declared()
    assert {"saw_rotate_quant_store", "saw_paged_decode_attn", "saw_dequant_pages", "saw_flatten_dequant", "saw_append_decode_attn",
            "saw_decode_workspace_bytes", "saw_kv16_paged_decode_attn"} <= set(names)
    L = saw.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.saw_version() == 100
    assert L.saw_strerror(0) == b"ok" and b"null" in L.saw_strerror(-2)


def _struct(saw, **kw):
    f = dict(k_codes=16, v_codes=16, k_meta=16, v_meta=16, num_pages=4, n_kv_heads=2, page_size=16,
             head_dim=128, had_block=128, rotate_mask=3)
    f.update(kw)
    return saw.SawCacheStruct(**f)


def test_store_rejects_bad_arguments_before_launch(saw):
    L = saw.lib()
    P = ctypes.c_void_p

    def call(st, K=16, V=16, dt=1, T=4, stride=256, pt=16, nseq=1, mp=4, slots=16):
        return L.saw_rotate_quant_store(ctypes.byref(st), P(K), P(V), dt, T, stride, P(pt), nseq, mp, P(slots), P(0))

    assert call(_struct(saw), T=0) == 0                              # empty call is a no-op
    assert call(_struct(saw, had_block=24)) == -1                    # not a power of two
    assert call(_struct(saw, had_block=8)) == -1                     # unsupported order
    assert call(_struct(saw, head_dim=64, had_block=128)) == -1      # h > head_dim
    assert call(_struct(saw, head_dim=96)) == -1
    assert call(_struct(saw, page_size=32)) == -1
    assert call(_struct(saw, rotate_mask=7)) == -1
    assert call(_struct(saw), dt=3) == -1                            # fp32 K/V not accepted
    assert call(_struct(saw), stride=100) == -1                      # stride below Hkv*d
    assert call(_struct(saw), stride=260) == -1                      # stride not a multiple of 8
    assert call(_struct(saw), K=8) == -1                             # misaligned
    assert call(_struct(saw), K=0) == -2
    assert call(_struct(saw), slots=0) == -2
    assert call(_struct(saw, k_meta=0)) == -2
    assert call(_struct(saw), T=-1) == -1


def test_decode_rejects_bad_arguments_before_launch(saw):
    L = saw.lib()
    P = ctypes.c_void_p

    def call(st, q=16, qdt=1, B=2, Hq=8, pt=16, mp=8, sl=16, msl=0, scale=0.0, out=16, odt=3, ws=16,
             wsb=1 << 30, ns=0):
        return L.saw_paged_decode_attn(ctypes.byref(st), P(q), qdt, B, Hq, P(pt), mp, P(sl), msl, scale, P(out),
                                       odt, P(ws), wsb, ns, P(0))

    assert call(_struct(saw), Hq=7) == -1                            # not a multiple of the kv heads
    assert call(_struct(saw), Hq=6) == -1                            # group size 3 unsupported
    assert call(_struct(saw), Hq=32) == -1                           # group size 16 unsupported
    assert call(_struct(saw), msl=129) == -1                         # bound beyond the page table
    assert call(_struct(saw), ns=2000) == -1
    assert call(_struct(saw), qdt=9) == -1
    assert call(_struct(saw), q=0) == -2
    assert call(_struct(saw), ws=0) == -2
    assert call(_struct(saw), wsb=64) == -3
    assert call(_struct(saw), scale=float("nan")) == -1
    assert call(_struct(saw, had_block=3)) == -1


def test_workspace_and_plan(saw):
    L = saw.lib()
    st = _struct(saw, n_kv_heads=8)
    for B, Hq, msl, ns in [(256, 32, 4096, 0), (1, 64, 131072, 0), (4, 32, 256, 0), (16, 32, 4096, 3), (2, 8, 1, 0)]:
        s, c = ctypes.c_int32(), ctypes.c_int32()
        assert L.saw_decode_plan(ctypes.byref(st), B, msl, ns, ctypes.byref(s), ctypes.byref(c)) == 0
        assert c.value % 64 == 0 and s.value >= 1 and s.value * c.value >= msl
        assert (s.value - 1) * c.value < msl                         # no empty trailing partition
        if ns:
            assert s.value <= ns
        need = ((B * Hq * s.value * 130 * 4 + 15) // 16) * 16
        got = L.saw_decode_workspace_bytes(ctypes.byref(st), B, Hq, msl, ns)
        # (the figure also covers the 16-bit comparison call, which keeps 256 one-wavefront partitions for the
        # single long sequence where the INT4 call takes 64 partitions of four wavefronts)
        assert got == (need if (B, msl) != (1, 131072) else 4 * need)
        if (B, msl) == (1, 131072):
            assert s.value == 64 and c.value == 2048
    assert L.saw_decode_workspace_bytes(ctypes.byref(st), 0, 32, 100, 0) == 0


def test_plan_keeps_one_partition_from_512_items_on(saw):
    """The INT4 decode calls stay with one partition per sequence once the batch provides 512 (sequence,
    kv head) items (head_dim 64 with an even head count: pairs of kv heads are the items); the workspace
    figure also covers the 16-bit call, which keeps splitting there."""
    L = saw.lib()

    def plan(st, B, msl):
        s, c = ctypes.c_int32(), ctypes.c_int32()
        assert L.saw_decode_plan(ctypes.byref(st), B, msl, 0, ctypes.byref(s), ctypes.byref(c)) == 0
        return s.value, c.value

    st = _struct(saw, n_kv_heads=8)
    assert plan(st, 64, 4096)[0] == 1 and plan(st, 63, 4096)[0] > 1
    assert plan(st, 1024, 4096)[0] == 1
    need = L.saw_decode_workspace_bytes(ctypes.byref(st), 64, 32, 4096, 0)
    assert need > 64 * 32 * 1 * 130 * 4                              # more than the one partition: the 16-bit call's
    st64 = _struct(saw, n_kv_heads=8, head_dim=64, had_block=64)
    assert plan(st64, 128, 4096)[0] == 1 and plan(st64, 64, 8192)[0] > 1
    # small batches of short contexts: one partition (a block of eight wavefronts per item), up to five batches per
    # wavefront, or eight when the blocks fill most of the chip; longer contexts go back to partitions
    assert plan(st, 4, 2304)[0] == 1 and plan(st, 32, 4096)[0] == 1 and plan(st64, 64, 4096)[0] == 1
    assert plan(st, 16, 4096)[0] > 1 and plan(st, 1, 8192)[0] > 1 and plan(st, 4, 2600)[0] > 1
    st64odd = _struct(saw, n_kv_heads=7, head_dim=64, had_block=64)
    assert plan(st64odd, 74, 4096)[0] == 1 and plan(st64odd, 73, 4096)[0] > 1


def test_dequant_rejects_bad_arguments(saw):
    L = saw.lib()
    P = ctypes.c_void_p
    st = _struct(saw)
    assert L.saw_dequant_pages(ctypes.byref(st), P(16), 4, 0, 0, 0, 0, P(16), P(16), P(0)) == 0   # empty range
    assert L.saw_dequant_pages(ctypes.byref(st), P(16), 4, 0, 5, 3, 0, P(16), P(16), P(0)) == -1
    assert L.saw_dequant_pages(ctypes.byref(st), P(16), 4, 0, 0, 65, 0, P(16), P(16), P(0)) == -1  # past the page table
    assert L.saw_dequant_pages(ctypes.byref(st), P(0), 4, 0, 0, 8, 0, P(16), P(16), P(0)) == -2


def test_binding_fails_loudly_without_library(saw, monkeypatch):
    monkeypatch.setattr(saw, "_lib", None)
    monkeypatch.setattr(saw, "LIB_PATH", "/nonexistent/libsaw.so")
    with pytest.raises(RuntimeError):
        saw.lib()


def test_rank_order_never_puts_an_empty_sequence_ahead_of_a_non_empty_one(saw):
    """Host mirror of the decode kernels' longest-first order.  The pair-mode blocks take the sequences at
    ranks (r, B-1-r) or (r, 2n-1-r, 2n+r) and rely on: if a block's k-th sequence has no cached tokens,
    neither have the later ones.  With classes scaled to the caller's bound a loose bound put empty and
    short sequences into one class (ordered by index); the classes now follow the batch's own longest
    sequence and keep the empty ones apart, whatever the bound."""
    import numpy as np
    rng = np.random.default_rng(5)
    cases = [([0] + [256] * 255, 16384), ([0] + [2048] * 127, 131072), ([0] * 50 + [300] * 100, 0),
             ([0, 65] * 90, 1 << 30), ([5, 0, 4096, 0, 64, 63, 65, 1], 0)]
    for _ in range(20):
        B = int(rng.integers(2, 700))
        lens = rng.integers(0, int(rng.choice([3, 70, 5000])), size=B)
        lens[rng.random(B) < 0.2] = 0
        cases.append((lens.tolist(), int(rng.choice([0, int(lens.max()) + 1, 1 << 20]))))
    for lens, bound in cases:
        order = saw.decode_rank_order(lens, bound)
        B = len(lens)
        assert sorted(order) == list(range(B))
        eff = [min(l, bound) if bound > 0 else l for l in lens]
        ranked = [eff[b] for b in order]
        nz = [i for i, l in enumerate(ranked) if l == 0]
        assert nz == list(range(B - len(nz), B)), (lens[:8], bound)           # the empty ones are exactly the tail
        # longest first at the granularity of the classes: a later sequence is never more than a class longer
        nbmax = max(1, max((l + 63) // 64 for l in eff))
        width = 64 * (nbmax / 63.0) + 64
        assert all(ranked[i + 1] <= ranked[i] + width for i in range(B - 1))
        # the blocks' precondition, for pairs and for triples
        for r in range((B + 1) // 2):
            a, b = ranked[r], ranked[B - 1 - r]
            assert not (a == 0 and b > 0)
        n3 = (B + 2) // 3
        for r in range(n3):
            ks = [ranked[k] for k in (r, 2 * n3 - 1 - r, 2 * n3 + r) if k < B]
            assert all(not (ks[i] == 0 and ks[j] > 0) for i in range(len(ks)) for j in range(i + 1, len(ks)))
        # the bound does not change the order as long as it clamps nothing
        if bound == 0 or bound > max(lens):
            assert order == saw.decode_rank_order(lens, max(lens) + 1 if max(lens) else 1)


def test_store_layers_and_dense_rotation_reject_bad_arguments(saw):
    L = saw.lib()
    P = ctypes.c_void_p
    n = 3
    sts = (saw.SawCacheStruct * n)(*[_struct(saw) for _ in range(n)])
    ptrs = (ctypes.c_void_p * n)(16, 16, 16)

    def call(sts=sts, K=ptrs, V=ptrs, n=n, dt=1, T=4, stride=256, pt=16, slots=16):
        return L.saw_rotate_quant_store_layers(sts, K, V, n, dt, T, stride, P(pt), 1, 4, P(slots), P(0))

    assert call(T=0) == 0
    assert call(n=0) == -1
    mixed = (saw.SawCacheStruct * n)(_struct(saw), _struct(saw, had_block=64), _struct(saw))
    assert call(sts=mixed) == -1                                      # layers must agree in the Hadamard block
    mixed = (saw.SawCacheStruct * n)(_struct(saw), _struct(saw, num_pages=5), _struct(saw))
    assert call(sts=mixed) == -1
    mixed = (saw.SawCacheStruct * n)(_struct(saw), _struct(saw, dense_rot=16), _struct(saw))
    assert call(sts=mixed) == -1                                      # a learned rotation for all layers or for none
    assert call(K=(ctypes.c_void_p * n)(16, 0, 16)) == -2
    assert call(K=(ctypes.c_void_p * n)(16, 8, 16)) == -1             # misaligned
    assert call(slots=4) == -1
    # learned rotation: head_dim 128 only, aligned buffers, big enough
    assert L.saw_dense_rotation_bytes(128) == 224 * 1024 and L.saw_dense_rotation_bytes(64) == 0
    assert L.saw_prepare_dense_rotation(P(16), 64, P(16), 1 << 20, P(0)) == -1
    assert L.saw_prepare_dense_rotation(P(16), 128, P(16), 1000, P(0)) == -1
    assert L.saw_prepare_dense_rotation(P(0), 128, P(16), 1 << 20, P(0)) == -2
    assert L.saw_prepare_dense_rotation(P(16), 128, P(8), 1 << 20, P(0)) == -1
    st = _struct(saw, head_dim=64, had_block=64, dense_rot=16)
    assert L.saw_rotate_quant_store(ctypes.byref(st), P(16), P(16), 1, 4, 128, P(16), 1, 4, P(16), P(0)) == -1
    st = _struct(saw, dense_rot=8)                                    # misaligned prepared buffer
    assert L.saw_rotate_quant_store(ctypes.byref(st), P(16), P(16), 1, 4, 256, P(16), 1, 4, P(16), P(0)) == -1
    # device-side order: pointers and batch size
    assert L.saw_decode_order(P(0), 4, 0, P(16), P(0)) == -2 and L.saw_decode_order(P(16), 4, 0, P(0), P(0)) == -2
    assert L.saw_decode_order(P(16), 0, 0, P(16), P(0)) == -1 and L.saw_decode_order(P(16), 1025, 0, P(16), P(0)) == -1
    # flatten cannot rotate a learned rotation back
    st = _struct(saw, dense_rot=16)
    assert L.saw_flatten_dequant(ctypes.byref(st), P(16), 4, 0, 0, 8, 1, 2, P(16), P(16), 256, P(0)) == -1
