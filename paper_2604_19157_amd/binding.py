"""ctypes binding of the C ABI declared in ``include/saw.h``.

Argument marshalling only: torch supplies device memory and the current stream, every
step of the path runs in the HIP kernels of ``libsaw.so``.  There is no CPU fallback: if
the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsaw.so")

SAW_F16, SAW_BF16, SAW_F32 = 1, 2, 3
ROT_K, ROT_V = 1, 2
_DT = {torch.float16: SAW_F16, torch.bfloat16: SAW_BF16, torch.float32: SAW_F32}


class SawCacheStruct(ctypes.Structure):
    _fields_ = [("k_codes", ctypes.c_void_p), ("v_codes", ctypes.c_void_p),
                ("k_meta", ctypes.c_void_p), ("v_meta", ctypes.c_void_p),
                ("num_pages", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("had_block", ctypes.c_int32), ("rotate_mask", ctypes.c_int32),
                ("sign_bits", ctypes.c_uint32 * 4), ("dense_rot", ctypes.c_void_p)]


class SawHints(ctypes.Structure):
    _fields_ = [("order", ctypes.c_void_p)]


class SawError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().saw_strerror(code).decode()} ({code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load ``libsaw.so`` (built by ``__graft_entry__.build()``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
        cp = ctypes.POINTER(SawCacheStruct)
        L.saw_version.restype = ctypes.c_int
        L.saw_strerror.restype = ctypes.c_char_p
        L.saw_strerror.argtypes = [ctypes.c_int]
        L.saw_dense_rotation_bytes.restype = sz
        L.saw_dense_rotation_bytes.argtypes = [i32]
        L.saw_prepare_dense_rotation.argtypes = [vp, i32, vp, sz, vp]
        L.saw_rotate_quant_store.argtypes = [cp, vp, vp, i32, i64, i64, vp, i32, i32, vp, vp]
        L.saw_rotate_quant_store_layers.argtypes = [cp, ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i32, i64, i64, vp, i32,
                                                    i32, vp, vp]
        L.saw_decode_order.argtypes = [vp, i32, i32, vp, vp]
        L.saw_read_probe.argtypes = [cp, vp, i64, vp, sz, vp]
        L.saw_plain_quant_store_valu.argtypes = [cp, vp, vp, i32, i64, i64, vp, i32, i32, vp, vp]
        L.saw_decode_workspace_bytes.restype = sz
        L.saw_decode_workspace_bytes.argtypes = [cp, i32, i32, i32, i32]
        L.saw_decode_plan.argtypes = [cp, i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.saw_decode_rank_order.argtypes = [ctypes.POINTER(i32), i32, i32, ctypes.POINTER(i32)]
        L.saw_paged_decode_attn.argtypes = [cp, vp, i32, i32, i32, vp, i32, vp, i32, f32, vp, i32, vp, sz, i32, vp]
        L.saw_paged_decode_attn_static.argtypes = [cp, vp, i32, i32, i32, vp, i32, vp, i32, f32, vp, i32, i32, vp]
        hp = ctypes.POINTER(SawHints)
        L.saw_paged_decode_attn_hinted.argtypes = [cp, vp, i32, i32, i32, vp, i32, vp, i32, f32, vp, i32, vp, sz, i32, hp, vp]
        L.saw_append_decode_attn_hinted.argtypes = [cp, vp, vp, i32, vp, i32, i32, i32, vp, i32, vp, i32, f32, vp, i32, vp, sz,
                                                    hp, vp]
        L.saw_dequant_pages.argtypes = [cp, vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.saw_append_decode_attn.argtypes = [cp, vp, vp, i32, vp, i32, i32, i32, vp, i32, vp, i32, f32, vp, i32, vp, sz, vp]
        L.saw_flatten_dequant.argtypes = [cp, vp, i32, i32, i32, i32, i32, i32, vp, vp, ctypes.c_int64, vp]
        L.saw_kv16_store.argtypes = [cp, vp, vp, i32, vp, vp, i64, i64, vp, i32, i32, vp, vp]
        L.saw_kv16_paged_decode_attn.argtypes = [cp, vp, vp, i32, vp, i32, i32, i32, vp, i32, vp, i32, f32,
                                                 vp, i32, vp, sz, i32, vp]
        _lib = L
    return _lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _check(code: int, where: str):
    if code != 0:
        raise SawError(code, where)


class Cache:
    """One layer's INT4 paged cache: device tensors plus the shape/rotation descriptor."""

    def __init__(self, num_pages, n_kv_heads, head_dim, had_block, rotate_mask=ROT_K | ROT_V,
                 page_size=16, device="cuda", zero=True, signs=None, dense=None):
        alloc = torch.zeros if zero else torch.empty
        self.k_codes = alloc((num_pages, n_kv_heads, page_size, head_dim // 2), dtype=torch.uint8, device=device)
        self.v_codes = alloc((num_pages, n_kv_heads, page_size, head_dim // 2), dtype=torch.uint8, device=device)
        self.k_meta = alloc((num_pages, n_kv_heads, page_size, 2), dtype=torch.float32, device=device)
        self.v_meta = alloc((num_pages, n_kv_heads, page_size, 2), dtype=torch.float32, device=device)
        self.num_pages, self.n_kv_heads, self.page_size = num_pages, n_kv_heads, page_size
        self.head_dim, self.had_block, self.rotate_mask = head_dim, had_block, rotate_mask
        # signs: head_dim values of +1 / -1 (the diagonal in front of the Hadamard matrix), or None
        self.sign_bits = [0, 0, 0, 0]
        if signs is not None:
            assert len(signs) == head_dim
            for c, v in enumerate(signs):
                if v < 0:
                    self.sign_bits[c // 32] |= 1 << (c % 32)

        # dense: the learned rotation R_l, a [head_dim][head_dim] array-like (y = x R_l), or None
        self.dense_rot = prepare_dense_rotation(dense, head_dim, device) if dense is not None else None

    def struct(self) -> SawCacheStruct:
        return SawCacheStruct(self.k_codes.data_ptr(), self.v_codes.data_ptr(), self.k_meta.data_ptr(),
                              self.v_meta.data_ptr(), self.num_pages, self.n_kv_heads, self.page_size,
                              self.head_dim, self.had_block, self.rotate_mask,
                              (ctypes.c_uint32 * 4)(*self.sign_bits),
                              self.dense_rot.data_ptr() if self.dense_rot is not None else None)

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.k_codes, self.v_codes, self.k_meta, self.v_meta))


def prepare_dense_rotation(R, head_dim, device="cuda"):
    """saw_prepare_dense_rotation: R ``[d][d]`` (array-like or tensor, y = x R) -> the prepared device buffer."""
    Rt = torch.as_tensor(R, dtype=torch.float32).to(device).contiguous()
    assert Rt.shape == (head_dim, head_dim)
    n = lib().saw_dense_rotation_bytes(head_dim)
    if n == 0:
        raise SawError(-1, "saw_dense_rotation_bytes")
    buf = torch.empty(n, dtype=torch.uint8, device=device)
    _check(lib().saw_prepare_dense_rotation(_ptr(Rt), head_dim, _ptr(buf), n, _stream()), "saw_prepare_dense_rotation")
    return buf


def rotate_quant_store(cache: Cache, K, V, page_table, slots):
    """saw_rotate_quant_store: K, V ``[T][Hkv][d]`` fp16/bf16, page_table ``[n_seqs][max_pages]`` int32,
    slots ``[T][2]`` int32, all on the device."""
    T = K.shape[0]
    assert K.dtype == V.dtype and K.shape == V.shape and K.stride(2) == 1 and K.stride(1) == cache.head_dim
    assert V.stride() == K.stride() and page_table.dtype == torch.int32 and slots.dtype == torch.int32
    assert page_table.is_contiguous() and slots.is_contiguous() and slots.shape == (T, 2)
    st = cache.struct()
    _check(lib().saw_rotate_quant_store(ctypes.byref(st), _ptr(K), _ptr(V), _DT[K.dtype], T,
                                        K.stride(0) if T > 1 else cache.n_kv_heads * cache.head_dim,
                                        _ptr(page_table), page_table.shape[0], page_table.shape[1],
                                        _ptr(slots), _stream()), "saw_rotate_quant_store")


def rotate_quant_store_layers(caches, Ks, Vs, page_table, slots):
    """saw_rotate_quant_store_layers: lists of n_layers caches and ``[T][Hkv][d]`` K / V tensors, one launch
    per 32 layers."""
    n = len(caches)
    c0 = caches[0]
    T = Ks[0].shape[0]
    stride = Ks[0].stride(0) if T > 1 else c0.n_kv_heads * c0.head_dim
    for K, V in zip(Ks, Vs):
        assert K.dtype == Ks[0].dtype and K.shape == Ks[0].shape == V.shape and K.stride(2) == 1 and K.stride(1) == c0.head_dim
        assert V.stride() == K.stride() and (T <= 1 or K.stride(0) == stride)
    assert len(Ks) == n == len(Vs) and page_table.is_contiguous() and slots.is_contiguous() and slots.shape == (T, 2)
    sts = (SawCacheStruct * n)(*[c.struct() for c in caches])
    kp = (ctypes.c_void_p * n)(*[K.data_ptr() for K in Ks])
    vp_ = (ctypes.c_void_p * n)(*[V.data_ptr() for V in Vs])
    _check(lib().saw_rotate_quant_store_layers(sts, kp, vp_, n, _DT[Ks[0].dtype], T, stride, _ptr(page_table),
                                               page_table.shape[0], page_table.shape[1], _ptr(slots), _stream()),
           "saw_rotate_quant_store_layers")


def decode_order(seq_lens, max_seq_len=0):
    """saw_decode_order: the longest-first order of the batch, computed on the device (int32 device tensors)."""
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous()
    order = torch.empty_like(seq_lens)
    _check(lib().saw_decode_order(_ptr(seq_lens), seq_lens.numel(), int(max_seq_len), _ptr(order), _stream()),
           "saw_decode_order")
    return order


def read_probe(cache: Cache, page_ids, sink=None):
    """saw_read_probe: read-only walk over `page_ids` (int32 device tensor) in the decode kernel's pattern;
    returns the bytes it reads."""
    assert page_ids.dtype == torch.int32 and page_ids.is_contiguous()
    if sink is None:
        sink = torch.empty(2048, dtype=torch.int32, device=page_ids.device)
    st = cache.struct()
    _check(lib().saw_read_probe(ctypes.byref(st), _ptr(page_ids), page_ids.numel(), _ptr(sink), sink.numel() * 4,
                                _stream()), "saw_read_probe")
    return page_ids.numel() * cache.n_kv_heads * 2304


def plain_quant_store_valu(cache: Cache, K, V, page_table, slots):
    """saw_plain_quant_store_valu: the plain INT4 store on the vector ALU (comparator; head_dim 128)."""
    T = K.shape[0]
    assert K.dtype == V.dtype and K.shape == V.shape and K.stride(2) == 1 and K.stride(1) == cache.head_dim
    st = cache.struct()
    _check(lib().saw_plain_quant_store_valu(ctypes.byref(st), _ptr(K), _ptr(V), _DT[K.dtype], T,
                                            K.stride(0) if T > 1 else cache.n_kv_heads * cache.head_dim,
                                            _ptr(page_table), page_table.shape[0], page_table.shape[1], _ptr(slots),
                                            _stream()), "saw_plain_quant_store_valu")


def decode_workspace_bytes(cache: Cache, B, n_q_heads, max_seq_len, num_splits=0) -> int:
    st = cache.struct()
    return int(lib().saw_decode_workspace_bytes(ctypes.byref(st), B, n_q_heads, max_seq_len, num_splits))


def decode_plan(cache: Cache, B, max_seq_len, num_splits=0):
    st = cache.struct()
    s, c = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().saw_decode_plan(ctypes.byref(st), B, max_seq_len, num_splits, ctypes.byref(s), ctypes.byref(c)),
           "saw_decode_plan")
    return s.value, c.value


def decode_rank_order(seq_lens, max_seq_len=0):
    """saw_decode_rank_order: host-side mirror of the decode kernels' longest-first order (host ints in, list out)."""
    B = len(seq_lens)
    src = (ctypes.c_int32 * B)(*[int(x) for x in seq_lens])
    dst = (ctypes.c_int32 * B)()
    _check(lib().saw_decode_rank_order(src, B, int(max_seq_len), dst), "saw_decode_rank_order")
    return list(dst)


def paged_decode_attn(cache: Cache, q, page_table, seq_lens, max_seq_len=0, sm_scale=0.0, out=None,
                      out_dtype=torch.float32, workspace=None, num_splits=0, order=None):
    """saw_paged_decode_attn: q ``[B][Hq][d]``; returns ``out [B][Hq][d]``.  With ``order`` (int32 device
    tensor, the sequences longest first) the call is saw_paged_decode_attn_hinted."""
    B, Hq, d = q.shape
    assert q.is_contiguous() and page_table.is_contiguous() and seq_lens.dtype == torch.int32
    bound = max_seq_len if max_seq_len > 0 else page_table.shape[1] * cache.page_size
    if out is None:
        out = torch.empty((B, Hq, d), dtype=out_dtype, device=q.device)
    need = decode_workspace_bytes(cache, B, Hq, bound, num_splits)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    st = cache.struct()
    if order is not None:
        assert order.dtype == torch.int32 and order.numel() == B and order.is_contiguous()
        hints = SawHints(order.data_ptr())
        _check(lib().saw_paged_decode_attn_hinted(ctypes.byref(st), _ptr(q), _DT[q.dtype], B, Hq, _ptr(page_table),
                                                  page_table.shape[1], _ptr(seq_lens), max_seq_len, float(sm_scale),
                                                  _ptr(out), _DT[out.dtype], _ptr(workspace), workspace.numel(),
                                                  num_splits, ctypes.byref(hints), _stream()), "saw_paged_decode_attn_hinted")
        return out
    _check(lib().saw_paged_decode_attn(ctypes.byref(st), _ptr(q), _DT[q.dtype], B, Hq, _ptr(page_table),
                                       page_table.shape[1], _ptr(seq_lens), max_seq_len, float(sm_scale),
                                       _ptr(out), _DT[out.dtype], _ptr(workspace), workspace.numel(),
                                       num_splits, _stream()), "saw_paged_decode_attn")
    return out


def paged_decode_attn_static(cache: Cache, q, page_table, seq_lens, out, max_seq_len=0, sm_scale=0.0, num_splits=0):
    """saw_paged_decode_attn_static: the no-allocation variant (library-held scratch); `out` is the caller's."""
    B, Hq, d = q.shape
    assert q.is_contiguous() and page_table.is_contiguous() and seq_lens.dtype == torch.int32
    assert out.shape == (B, Hq, d) and out.is_contiguous()
    st = cache.struct()
    _check(lib().saw_paged_decode_attn_static(ctypes.byref(st), _ptr(q), _DT[q.dtype], B, Hq, _ptr(page_table),
                                              page_table.shape[1], _ptr(seq_lens), max_seq_len, float(sm_scale),
                                              _ptr(out), _DT[out.dtype], num_splits, _stream()),
           "saw_paged_decode_attn_static")
    return out


def append_decode_attn(cache: Cache, K_new, V_new, q, page_table, seq_lens, max_seq_len=0, sm_scale=0.0, out=None,
                       out_dtype=torch.float32, workspace=None, order=None):
    """saw_append_decode_attn: K_new, V_new ``[B][Hkv][d]`` (token b -> sequence b at position
    seq_lens[b]), q ``[B][Hq][d]``; stores the tokens and returns ``out [B][Hq][d]`` of the attention
    over seq_lens[b] + 1 tokens.  seq_lens (tokens cached before the call) is not modified."""
    B, Hq, d = q.shape
    assert q.is_contiguous() and K_new.is_contiguous() and V_new.is_contiguous() and K_new.dtype == V_new.dtype
    assert page_table.is_contiguous() and seq_lens.dtype == torch.int32
    cap = page_table.shape[1] * cache.page_size
    after = (max_seq_len if max_seq_len > 0 else cap - 1) + 1
    if out is None:
        out = torch.empty((B, Hq, d), dtype=out_dtype, device=q.device)
    need = decode_workspace_bytes(cache, B, Hq, after, 0)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    st = cache.struct()
    if order is not None:
        assert order.dtype == torch.int32 and order.numel() == B and order.is_contiguous()
        hints = SawHints(order.data_ptr())
        _check(lib().saw_append_decode_attn_hinted(ctypes.byref(st), _ptr(K_new), _ptr(V_new), _DT[K_new.dtype], _ptr(q),
                                                   _DT[q.dtype], B, Hq, _ptr(page_table), page_table.shape[1], _ptr(seq_lens),
                                                   max_seq_len, float(sm_scale), _ptr(out), _DT[out.dtype], _ptr(workspace),
                                                   workspace.numel(), ctypes.byref(hints), _stream()),
               "saw_append_decode_attn_hinted")
        return out
    _check(lib().saw_append_decode_attn(ctypes.byref(st), _ptr(K_new), _ptr(V_new), _DT[K_new.dtype], _ptr(q),
                                        _DT[q.dtype], B, Hq, _ptr(page_table), page_table.shape[1], _ptr(seq_lens),
                                        max_seq_len, float(sm_scale), _ptr(out), _DT[out.dtype], _ptr(workspace),
                                        workspace.numel(), _stream()), "saw_append_decode_attn")
    return out


def dequant_pages(cache: Cache, page_table, seq, pos_begin, pos_end, unrotate=False, want_k=True, want_v=True):
    """saw_dequant_pages: returns fp32 ``(K^, V^)`` each ``[n][Hkv][d]`` (None if not requested)."""
    n = pos_end - pos_begin
    dev = cache.k_codes.device
    k = torch.empty((n, cache.n_kv_heads, cache.head_dim), dtype=torch.float32, device=dev) if want_k else None
    v = torch.empty((n, cache.n_kv_heads, cache.head_dim), dtype=torch.float32, device=dev) if want_v else None
    st = cache.struct()
    _check(lib().saw_dequant_pages(ctypes.byref(st), _ptr(page_table), page_table.shape[1], seq, pos_begin,
                                   pos_end, int(bool(unrotate)), _ptr(k), _ptr(v), _stream()), "saw_dequant_pages")
    return k, v


def flatten_dequant(cache: Cache, page_table, seq, pos_begin, pos_end, unrotate=True, out_dtype=torch.bfloat16,
                    want_k=True, want_v=True, k_out=None, v_out=None):
    """saw_flatten_dequant: ``(K^, V^)`` each ``[n][Hkv][d]`` of out_dtype (None if not requested)."""
    n = pos_end - pos_begin
    dev = cache.k_codes.device
    shape = (n, cache.n_kv_heads, cache.head_dim)
    if want_k and k_out is None:
        k_out = torch.empty(shape, dtype=out_dtype, device=dev)
    if want_v and v_out is None:
        v_out = torch.empty(shape, dtype=out_dtype, device=dev)
    ref = k_out if k_out is not None else v_out
    stride = ref.stride(0) if ref is not None and n > 0 else cache.n_kv_heads * cache.head_dim
    dt = _DT[ref.dtype] if ref is not None else _DT[out_dtype]
    st = cache.struct()
    _check(lib().saw_flatten_dequant(ctypes.byref(st), _ptr(page_table), page_table.shape[1], seq, pos_begin,
                                     pos_end, int(bool(unrotate)), dt, _ptr(k_out), _ptr(v_out), stride,
                                     _stream()), "saw_flatten_dequant")
    return k_out, v_out


class Kv16Cache:
    """The 16-bit comparison cache: pages ``[num_pages][Hkv][16][d]`` of fp16/bf16."""

    def __init__(self, num_pages, n_kv_heads, head_dim, dtype, page_size=16, device="cuda"):
        self.k_pages = torch.zeros((num_pages, n_kv_heads, page_size, head_dim), dtype=dtype, device=device)
        self.v_pages = torch.zeros((num_pages, n_kv_heads, page_size, head_dim), dtype=dtype, device=device)
        self.num_pages, self.n_kv_heads, self.page_size, self.head_dim = num_pages, n_kv_heads, page_size, head_dim
        self.dtype = dtype

    def struct(self) -> SawCacheStruct:
        return SawCacheStruct(0, 0, 0, 0, self.num_pages, self.n_kv_heads, self.page_size, self.head_dim, 1, 0)

    def nbytes(self) -> int:
        return 2 * self.k_pages.numel() * self.k_pages.element_size()


def kv16_store(cache: Kv16Cache, K, V, page_table, slots):
    T = K.shape[0]
    assert K.dtype == cache.dtype and V.dtype == cache.dtype and K.stride() == V.stride()
    st = cache.struct()
    _check(lib().saw_kv16_store(ctypes.byref(st), _ptr(cache.k_pages), _ptr(cache.v_pages), _DT[cache.dtype],
                                _ptr(K), _ptr(V), T, K.stride(0) if T > 1 else cache.n_kv_heads * cache.head_dim,
                                _ptr(page_table), page_table.shape[0], page_table.shape[1], _ptr(slots),
                                _stream()), "saw_kv16_store")


def kv16_paged_decode_attn(cache: Kv16Cache, q, page_table, seq_lens, max_seq_len=0, sm_scale=0.0, out=None,
                           out_dtype=torch.float32, workspace=None, num_splits=0):
    B, Hq, d = q.shape
    bound = max_seq_len if max_seq_len > 0 else page_table.shape[1] * cache.page_size
    if out is None:
        out = torch.empty((B, Hq, d), dtype=out_dtype, device=q.device)
    st = cache.struct()
    need = int(lib().saw_decode_workspace_bytes(ctypes.byref(st), B, Hq, bound, num_splits))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(lib().saw_kv16_paged_decode_attn(ctypes.byref(st), _ptr(cache.k_pages), _ptr(cache.v_pages),
                                            _DT[cache.dtype], _ptr(q), _DT[q.dtype], B, Hq, _ptr(page_table),
                                            page_table.shape[1], _ptr(seq_lens), max_seq_len, float(sm_scale),
                                            _ptr(out), _DT[out.dtype], _ptr(workspace), workspace.numel(),
                                            num_splits, _stream()), "saw_kv16_paged_decode_attn")
    return out
