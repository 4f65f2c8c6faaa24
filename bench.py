#!/usr/bin/env python3
"""Benchmark of the SAW-INT4 KV-cache hot path on one MI355X.

A step = one decode iteration of the high-concurrency workload (batch 256, context uniform in
[512, 4096], 32 query / 8 kv heads, head_dim 128, page 16, Hadamard block 64, bf16 inputs):
the fused rotate-quantise-store of the batch's 256 new tokens followed by the INT4 paged
decode attention over every cached token.  All inputs are resident in HBM before the timed
region.  Prints ONE JSON line (see the fields at the bottom of main()).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2604_19157_amd import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth


def progress(msg):
    """One line on stderr per finished stage of the run (the JSON line on stdout stays alone)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def profiled_traffic():
    """HBM bytes per decode launch from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE, scaled by the copy-kernel calibration written there); None if it is absent."""
    try:
        with open(os.path.join(ROOT, "profiles", "decode_int4_mfma_highconc.md")) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(line.split(":")[1])
    except OSError:
        pass
    return None


def decode_bytes(w, lens) -> int:
    """Algorithmic bytes of one decode call: codes + metadata of every cached token, page-table
    entries, q in and o out."""
    tok = int(np.asarray(lens, np.int64).sum())
    per_tok = w.n_kv_heads * (w.head_dim + 16)
    pt = int(sum((int(L) + 15) // 16 for L in lens)) * 4
    qo = len(lens) * w.n_q_heads * w.head_dim * (torch.finfo(w.dtype).bits // 8 + 4)
    return tok * per_tok + pt + qo


def kv16_decode_bytes(w, lens) -> int:
    tok = int(np.asarray(lens, np.int64).sum())
    pt = int(sum((int(L) + 15) // 16 for L in lens)) * 4
    qo = len(lens) * w.n_q_heads * w.head_dim * (2 + 4)
    return tok * w.n_kv_heads * w.head_dim * 4 + pt + qo


def store_bytes(w, T) -> int:
    return T * (2 * w.n_kv_heads * w.head_dim * 2 + w.n_kv_heads * (w.head_dim + 16))


def fill(w, saw, dev, cache, kv16=None, chunk=8192):
    pt = torch.from_numpy(w.page_table).to(dev)
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        for p0 in range(0, L, chunk):
            p1 = min(L, p0 + chunk)
            K, V = synth.gen_kv(w, b, p0, p1, device=dev)
            sl = torch.from_numpy(synth.slots_for(b, p0, p1)).to(dev)
            saw.rotate_quant_store(cache, K, V, pt, sl)
            if kv16 is not None:
                saw.kv16_store(kv16, K, V, pt, sl)
    torch.cuda.synchronize()
    return pt


SETTLE_S = 0.15              # untimed calls before every measurement: after an idle gap the clocks need ~0.1 s to come back up


# the side workloads are timed right after their caches are filled and cloned (the GPU has been doing
# other, lighter work): half a second of the call itself first, or the first figures come out 30-40 % slow
OTHER_SETTLE_S = 0.5


def _settle(fns, seconds):
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(8):
            for fn in fns:
                fn()
        torch.cuda.synchronize()


def time_calls(fn, iters, warmup, settle=SETTLE_S):
    """Median / mean of per-call durations measured with events on the current stream."""
    _settle([fn], settle)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = np.array([a.elapsed_time(b) for a, b in ev]) * 1e3     # us
    return float(np.median(ts)), float(ts.mean()), float(np.percentile(ts, 10)), float(np.percentile(ts, 90))


def time_interleaved(fns, iters, warmup, settle=SETTLE_S):
    """Median per-call duration (us) of each of several callables, called in turn (a, b, c, a, b, c ...)
    so that clock drift over the run hits all of them alike and their ratios stay meaningful."""
    _settle(fns, settle)
    for _ in range(warmup):
        for fn in fns:
            fn()
    torch.cuda.synchronize()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in fns] for _ in range(iters)]
    for row in ev:
        for fn, (a, b) in zip(fns, row):
            a.record()
            fn()
            b.record()
    torch.cuda.synchronize()
    ts = np.array([[a.elapsed_time(b) for a, b in row] for row in ev]) * 1e3
    return [float(x) for x in np.median(ts, axis=0)]


def cpu_baseline(w, budget_s=20.0):
    """The oracle as it stands, timed on the host on a bounded sample of the same workload:
    store + decode of the first sequences of the batch until ~budget_s of CPU time is used."""
    from oracle import saw_oracle as O
    t0 = time.perf_counter()
    nbytes = 0
    n_seq = 0
    tokens = 0
    spent = 0.0
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        sub = synth.make_workload(w.name, batch=1, seq_lens=[L])
        ref = O.new_cache(sub.num_pages, w.n_kv_heads, w.page_size, w.head_dim)
        K, V = synth.gen_kv(w, b, 0, L)
        Kf, Vf = K.float().numpy(), V.float().numpy()
        q = synth.gen_q(w)[b:b + 1].float().numpy()
        t1 = time.perf_counter()
        O.rotate_quant_store(ref, Kf, Vf, sub.page_table, synth.slots_for(0, 0, L), w.had_block, w.rotate_mask)
        O.paged_decode_attn(ref, q, sub.page_table, np.array([L], np.int32), w.had_block, w.rotate_mask)
        dt = time.perf_counter() - t1
        nbytes += store_bytes(w, L) + decode_bytes(w, [L])
        tokens += L
        n_seq += 1
        spent += dt
        if time.perf_counter() - t0 > budget_s:
            break
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": nbytes / spent / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "implementation": f"numpy fp64 (explicit matrices, two-pass softmax); its matrix products run on the BLAS "
                              f"pool, {int(cores)} threads; everything else is single-threaded",
            "sample": f"oracle store + decode of the first {n_seq} sequences ({tokens} tokens) of the workload, "
                      f"{spent:.1f} s of oracle time; bytes = same algorithmic bytes as the GPU figure"}


SWEEP_SETS = 8               # buffer sets a sweep rotates over (inputs 134 MB + cache 38 MB each: 8 sets = 5x the 256 MB memory-side cache)


def store_sweep(saw, dev, iters=30, warmup=5, same_buffers=True):
    """Prefill store, 32768-token chunk: tokens/s per Hadamard block size (1 = plain INT4).
    Every call takes the next of SWEEP_SETS (input, cache) sets, so neither the K/V read nor the
    pages written are still in the memory-side cache from the previous call ("us"); "us_same_buffers"
    is the same call repeated on one set, i.e. with the 134 MB input largely cache-resident."""
    out = {}
    for name in ("prefill", "prefill_mha"):
        res = {}
        base = synth.make_workload(name)
        T = int(base.seq_lens[0])
        K, V = synth.gen_kv(base, 0, 0, T, device=dev)
        Ks = [K] + [K.clone() for _ in range(SWEEP_SETS - 1)]
        Vs = [V] + [V.clone() for _ in range(SWEEP_SETS - 1)]
        pt = torch.from_numpy(base.page_table).to(dev)
        sl = torch.from_numpy(synth.slots_for(0, 0, T)).to(dev)
        # variants: every block size, plus the largest one with a random +/-1 diagonal in front of the
        # Hadamard matrix (randomised Hadamard, Sec. 3); all timed in turn (plain, 16, 32, ..., plain, 16, ...),
        # each call on the next buffer set
        # also: K-only rotation (the serving default of App. D: V stored as plain INT4), a learned per-layer
        # rotation after the Hadamard (App. A.3, a seeded random orthogonal matrix standing in for it), and - as
        # the leanest possible plain INT4 store - a vector-ALU kernel without matrix cores or LDS staging
        hmax = min(128, base.head_dim)
        variants = [(f"h{h}", h, None, 3, None) for h in (1, 16, 32, 64, 128) if h <= base.head_dim]
        variants.append((f"h{hmax}_signs", hmax, synth.random_signs(base.head_dim, 1), 3, None))
        variants.append((f"h{hmax}_k_only", hmax, None, 1, None))
        if base.head_dim == 128:
            variants.append(("h128_learned", 128, None, 3, synth.random_orthogonal(128, 2)))
            variants.append(("h1_valu", 1, None, 3, None))
        for h in (1, 16, 32, 64, 128):
            if h > base.head_dim:
                res[f"h{h}"] = None
        dense_bufs = {key: saw.prepare_dense_rotation(dn, base.head_dim, dev) for key, _, _, _, dn in variants if dn is not None}

        def new_cache(key, h, sg, mask):
            c = saw.Cache(base.num_pages, base.n_kv_heads, base.head_dim, h, mask, device=dev, signs=sg)
            c.dense_rot = dense_bufs.get(key)
            return c

        caches = {key: [new_cache(key, h, sg, mask) for _ in range(SWEEP_SETS)] for key, h, sg, mask, _ in variants}
        store_fn = lambda key: saw.plain_quant_store_valu if key == "h1_valu" else saw.rotate_quant_store

        def make_call(key):
            turn = [0]                                          # every variant walks all its buffer sets

            def call():
                i = turn[0] % SWEEP_SETS
                turn[0] += 1
                store_fn(key)(caches[key][i], Ks[i], Vs[i], pt, sl)
            return call

        meds = time_interleaved([make_call(v[0]) for v in variants], iters, warmup)
        sames = (time_interleaved([(lambda key=v[0]: store_fn(key)(caches[key][0], K, V, pt, sl)) for v in variants],
                                  iters, warmup) if same_buffers else [None] * len(variants))
        for (key, h, sg, mask, dn), med, same in zip(variants, meds, sames):
            if dn is not None:                                  # (the flatten call does not rotate a learned rotation back)
                res[key] = {"us": round(med, 2), "us_same_buffers": None if same is None else round(same, 2),
                            "Gtok_s": round(T / med / 1e3, 4), "GB_s": round(store_bytes(base, T) / med / 1e3, 1), "k_mse": None}
                continue
            # sanity column: quantisation error of K against the unquantised input (read back, rotated back)
            kq, _ = saw.flatten_dequant(caches[key][0], pt, 0, 0, T, unrotate=True, out_dtype=torch.float32, want_v=False)
            mse = float(((kq - K.float()) ** 2).mean())
            del kq
            res[key] = {"us": round(med, 2), "us_same_buffers": None if same is None else round(same, 2), "Gtok_s": round(T / med / 1e3, 4),
                        "GB_s": round(store_bytes(base, T) / med / 1e3, 1), "k_mse": float(f"{mse:.4e}")}
        del caches
        plain = res["h1"]["us"]
        for k, v in res.items():
            if v is not None:
                v["vs_plain"] = round(v["us"] / plain, 4)                   # plain = this kernel with an identity matrix
                if "h1_valu" in res:
                    v["vs_plain_valu"] = round(v["us"] / res["h1_valu"]["us"], 4)   # plain = the lean vector-ALU store
        out[name] = res
        del Ks, Vs
    return out


def flatten_sweep(saw, dev, iters=30, warmup=5, same_buffers=True):
    """Flatten-dequantise of a 32768-token sequence into dense bf16 K and V: tokens/s per Hadamard
    block size, rotated back (and, for comparison, left in the rotated space = plain dequantise).
    Calls rotate over SWEEP_SETS caches and 4 output sets, so the pages are read from HBM, not from the
    memory-side cache ("us"); "us_same_buffers" repeats one set (its 38 MB of pages stay cached)."""
    out = {}
    for name in ("prefill", "prefill_mha"):
        res = {}
        base = synth.make_workload(name)
        T = int(base.seq_lens[0])
        K, V = synth.gen_kv(base, 0, 0, T, device=dev)
        pt = torch.from_numpy(base.page_table).to(dev)
        sl = torch.from_numpy(synth.slots_for(0, 0, T)).to(dev)
        shape = (T, base.n_kv_heads, base.head_dim)
        kos = [torch.empty(shape, dtype=torch.bfloat16, device=dev) for _ in range(4)]
        vos = [torch.empty(shape, dtype=torch.bfloat16, device=dev) for _ in range(4)]
        nbytes = T * base.n_kv_heads * (2 * (base.head_dim // 2 + 8) + 2 * base.head_dim * 2)
        for h in (1, 16, 32, 64, 128):
            if h > base.head_dim:
                res[f"h{h}"] = None
                continue
            caches = [saw.Cache(base.num_pages, base.n_kv_heads, base.head_dim, h, 3, device=dev)
                      for _ in range(SWEEP_SETS)]
            for c in caches:
                saw.rotate_quant_store(c, K, V, pt, sl)
            r = {}
            for unrot in (True, False):
                turn = [0]

                def call():
                    i = turn[0] % SWEEP_SETS
                    turn[0] += 1
                    saw.flatten_dequant(caches[i], pt, 0, 0, T, unrotate=unrot, k_out=kos[i % 4], v_out=vos[i % 4])

                med, mean, p10, p90 = time_calls(call, iters, warmup)
                same = time_calls(lambda: saw.flatten_dequant(caches[0], pt, 0, 0, T, unrotate=unrot,
                                                              k_out=kos[0], v_out=vos[0]), iters, warmup)[0] if same_buffers else None
                r["rotated_back" if unrot else "as_stored"] = {"us": round(med, 2), "us_same_buffers": None if same is None else round(same, 2),
                                                               "Gtok_s": round(T / med / 1e3, 4),
                                                               "GB_s": round(nbytes / med / 1e3, 1)}
            r["rotation_cost"] = round(r["rotated_back"]["us"] / r["as_stored"]["us"], 4)
            res[f"h{h}"] = r
            del caches
        out[name] = res
    return out


LLC_BYTES = 256 << 20        # memory-side cache of the chip: smaller working sets are rotated over copies


def clone_cache(saw, c, dev):
    n = saw.Cache(c.num_pages, c.n_kv_heads, c.head_dim, c.had_block, c.rotate_mask, device=dev, zero=False)
    for k in ("k_codes", "v_codes", "k_meta", "v_meta"):
        getattr(n, k).copy_(getattr(c, k))
    return n


def other_decode(saw, dev, name, iters=32, warmup=8, with_kv16=False, with_append=False, **over):
    """Decode latency and bandwidth of another workload of the paper's table (cache filled by the HIP
    store).  A cache smaller than the chip's 256 MB memory-side cache would be served from it on
    repeated calls, so such workloads rotate over enough identical copies to exceed 4x that size.
    `with_kv16` adds the 16-bit-KV decode of the same workload, timed in turn with the INT4 one."""
    w = synth.make_workload(name, **over)
    cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask, device=dev)
    kv16 = saw.Kv16Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.dtype, device=dev) if with_kv16 else None
    pt = fill(w, saw, dev, cache, kv16)
    lens = w.seq_lens.astype(np.int32)
    nbytes = decode_bytes(w, lens)
    copies = [cache]
    while nbytes * len(copies) < 4 * LLC_BYTES and len(copies) < 16:
        copies.append(clone_cache(saw, cache, dev))
    seq_lens = torch.from_numpy(lens).to(dev)
    max_len = int(lens.max())
    q = synth.gen_q(w, device=dev)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device=dev)
    ws = torch.empty(saw.decode_workspace_bytes(cache, w.batch, w.n_q_heads, max_len), dtype=torch.uint8, device=dev)
    splits, chunk = saw.decode_plan(cache, w.batch, max_len)
    turn = [0]
    # the caller's longest-first order, as in the headline step (only read by the large-batch launch shapes)
    # (not when the 16-bit call, which has no such argument, is timed beside it: both then rank the batch themselves)
    order = torch.from_numpy(np.argsort(-lens, kind="stable").astype(np.int32)).to(dev) if (w.batch > 1 and not with_kv16) else None

    def call():
        c = copies[turn[0] % len(copies)]
        turn[0] += 1
        saw.paged_decode_attn(c, q, pt, seq_lens, max_seq_len=max_len, out=out, workspace=ws, order=order)

    res16 = None
    if with_kv16:
        def call16():
            saw.kv16_paged_decode_attn(kv16, q, pt, seq_lens, max_seq_len=max_len, out=out, workspace=ws)
        med, med16 = time_interleaved([call, call16], iters, warmup, settle=OTHER_SETTLE_S)
        p10 = p90 = float("nan")
        b16 = kv16_decode_bytes(w, lens)
        res16 = {"us": round(med16, 2), "GB_s": round(b16 / med16 / 1e3, 1), "int4_speedup": round(med16 / med, 3),
                 "bytes_ratio": round(b16 / nbytes, 3)}
    else:
        med, mean, p10, p90 = time_calls(call, iters, warmup, settle=OTHER_SETTLE_S)
    step_us = None
    if with_append:
        # the whole decode step: this step's token of every sequence appended and attended to, one call
        newK = torch.cat([synth.gen_kv(w, b, int(lens[b]), int(lens[b]) + 1, device=dev)[0] for b in range(w.batch)])
        newV = torch.cat([synth.gen_kv(w, b, int(lens[b]), int(lens[b]) + 1, device=dev)[1] for b in range(w.batch)])
        ws2 = torch.empty(saw.decode_workspace_bytes(cache, w.batch, w.n_q_heads, max_len + 1), dtype=torch.uint8, device=dev)

        def call_step():
            c = copies[turn[0] % len(copies)]
            turn[0] += 1
            saw.append_decode_attn(c, newK, newV, q, pt, seq_lens, max_seq_len=max_len, out=out, workspace=ws2, order=order)

        step_us = time_calls(call_step, iters, warmup, settle=OTHER_SETTLE_S)[0]
    overhead = 2 * w.batch * w.n_q_heads * splits * (w.head_dim + 2) * 4 if splits > 1 else 0
    r = {"batch": w.batch, "tokens_cached": int(lens.sum()), "splits": splits, "cache_copies_rotated": len(copies),
         "split_partials_bytes_written_and_read": overhead,
         "us": round(med, 2), "GB_s": round(nbytes / med / 1e3, 1),
         "pct_of_hbm_peak": round(nbytes / med / 1e3 / HBM_PEAK_GBS * 100, 2)}
    if step_us is not None:
        r["append_decode_step_us"] = round(step_us, 2)
    if res16 is None:
        r.update(p10_us=round(p10, 2), p90_us=round(p90, 2))
    else:
        r["kv16_decode"] = res16
    return r


def read_ceiling(saw, dev, w, cache, iters=30):
    """Read-only streaming ceiling of this machine for the decode kernel's access pattern: saw_read_probe walks the
    workload's pages (every sequence's pages in order, i.e. shuffled over the pool) and, for comparison, the
    same number of pages in address order.  GB/s of bytes read."""
    P = w.page_size
    ids = np.concatenate([w.page_table[b, :(int(w.seq_lens[b]) + P - 1) // P] for b in range(w.batch)]).astype(np.int32)
    shuffled = torch.from_numpy(ids).to(dev)
    ordered = torch.arange(len(ids), dtype=torch.int32, device=dev)
    sink = torch.empty(2048, dtype=torch.int32, device=dev)
    out = {}
    for key, pages in (("decode_pattern", shuffled), ("contiguous", ordered)):
        nbytes = saw.read_probe(cache, pages, sink)
        med = time_calls(lambda: saw.read_probe(cache, pages, sink), iters, 5)[0]
        out[key] = {"us": round(med, 2), "GB_s": round(nbytes / med / 1e3, 1), "pct_of_hbm_peak": round(nbytes / med / 1e3 / HBM_PEAK_GBS * 100, 2)}
    out["what"] = ("saw_read_probe: 2048 single-wavefront blocks reading the cache's K/V code tiles (1 KiB pieces) and "
                   "(scale, zero) pairs of the workload's pages, one 9 KiB batch ahead, nothing else")
    return out


def layers_store(saw, dev, n_layers=32, iters=50):
    """The decode step's KV write for a whole model: 16 new tokens (llama8b shape) for n_layers layers as one
    saw_rotate_quant_store_layers launch against n_layers saw_rotate_quant_store launches."""
    w = synth.make_workload("llama8b")
    caches = [saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask, device=dev) for _ in range(n_layers)]
    Ks = [torch.cat([synth.gen_kv(w, b + 100 * l, 4096, 4097, device=dev)[0] for b in range(w.batch)]) for l in range(n_layers)]
    Vs = [torch.cat([synth.gen_kv(w, b + 100 * l, 4096, 4097, device=dev)[1] for b in range(w.batch)]) for l in range(n_layers)]
    pt = torch.from_numpy(w.page_table).to(dev)
    sl = torch.from_numpy(np.stack([np.arange(w.batch, dtype=np.int32), np.full(w.batch, 4096, np.int32)], 1)).to(dev)

    def one_launch():
        saw.rotate_quant_store_layers(caches, Ks, Vs, pt, sl)

    def per_layer():
        for c, K, V in zip(caches, Ks, Vs):
            saw.rotate_quant_store(c, K, V, pt, sl)

    a = time_calls(one_launch, iters, 5)[0]
    b = time_calls(per_layer, iters, 5)[0]
    return {"layers": n_layers, "tokens_per_layer": w.batch, "one_launch_us": round(a, 2), "one_launch_us_per_layer": round(a / n_layers, 3),
            "per_layer_launches_us": round(b, 2), "per_layer_launches_us_per_layer": round(b / n_layers, 3)}


def copy_ceiling(dev, nbytes=1 << 30, iters=10):
    """On-box streaming ceiling: a plain device-to-device copy of 1 GiB (bytes read + bytes written per second)."""
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    med, mean, p10, p90 = time_calls(lambda: dst.copy_(src), iters, 3)
    del src, dst
    torch.cuda.empty_cache()
    return 2 * nbytes / med / 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-seconds", type=float, default=0.5,
                    help="untimed steps run for this long before the warm-up steps, so that clocks have settled")
    ap.add_argument("--no-extras", action="store_true", help="skip the kv16 / store-sweep / other-config figures")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-order-hint", action="store_true",
                    help="let the decode kernels rank the sequences by length themselves instead of handing them the "
                         "longest-first order (saw_append_decode_attn instead of saw_append_decode_attn_hinted)")
    ap.add_argument("--workload", default="highconc")
    ap.add_argument("--num-splits", type=int, default=0, help="split-KV factor (0 = the library's choice)")
    ap.add_argument("--store-sweep-only", action="store_true",
                    help="only run the prefill store sweep (32768-token chunk, every Hadamard block size, rotating "
                         "buffer sets only) and print it")
    ap.add_argument("--flatten-sweep-only", action="store_true",
                    help="only run the flatten-dequantise sweep (32768 tokens, every Hadamard block size, rotating "
                         "buffer sets only) and print it")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "reads": n, "writes": n, "repeats": 5}))
        return
    from paper_2604_19157_amd import binding as saw
    saw.lib()
    if args.store_sweep_only:
        print(json.dumps({"prefill_store_sweep": store_sweep(saw, dev, iters=args.steps, warmup=args.warmup, same_buffers=False)}))
        return

    if args.flatten_sweep_only:
        print(json.dumps({"prefill_flatten_sweep": flatten_sweep(saw, dev, iters=args.steps, warmup=args.warmup, same_buffers=False)}))
        return

    w = synth.make_workload(args.workload)
    B = w.batch
    cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask, device=dev)
    extras = not args.no_extras
    kv16 = saw.Kv16Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.dtype, device=dev) if extras else None
    pt = fill(w, saw, dev, cache, kv16)

    # the decode step's new tokens: one per sequence at position L_b (written every step)
    newK = torch.cat([synth.gen_kv(w, b, int(w.seq_lens[b]), int(w.seq_lens[b]) + 1, device=dev)[0] for b in range(B)])
    newV = torch.cat([synth.gen_kv(w, b, int(w.seq_lens[b]), int(w.seq_lens[b]) + 1, device=dev)[1] for b in range(B)])
    new_slots = torch.from_numpy(np.stack([np.arange(B, dtype=np.int32), w.seq_lens.astype(np.int32)], 1)).to(dev)
    lens0 = w.seq_lens.astype(np.int32)
    lens1 = (w.seq_lens + 1).astype(np.int32)
    seq_lens0 = torch.from_numpy(lens0).to(dev)
    seq_lens = torch.from_numpy(lens1).to(dev)
    max_len0 = int(lens0.max())
    max_len = int(lens1.max())
    q = synth.gen_q(w, device=dev)
    out = torch.empty((B, w.n_q_heads, w.head_dim), dtype=torch.float32, device=dev)
    ws = torch.empty(saw.decode_workspace_bytes(cache, B, w.n_q_heads, max_len, args.num_splits), dtype=torch.uint8, device=dev)
    splits, chunk = saw.decode_plan(cache, B, max_len, args.num_splits)
    fused = args.num_splits == 0
    # The longest-first order of the batch: computed once per decode step (it depends on the lengths only, so one
    # order serves the attention calls of all layers of the step), here on the device by saw_decode_order from the
    # device-resident lengths; handed to the call like the page table is.  Its own cost is in extra.decode_order_us.
    order = None if args.no_order_hint else saw.decode_order(seq_lens0, max_len0)

    def store_step():
        saw.rotate_quant_store(cache, newK, newV, pt, new_slots)

    def decode_step():
        saw.paged_decode_attn(cache, q, pt, seq_lens, max_seq_len=max_len, out=out, workspace=ws, num_splits=args.num_splits,
                              order=order)

    def fused_step():
        # one call (one kernel launch for this workload): append the step's tokens and attend over all of them
        saw.append_decode_attn(cache, newK, newV, q, pt, seq_lens0, max_seq_len=max_len0, out=out, workspace=ws, order=order)

    def step():
        if fused:
            fused_step()
        else:
            store_step()
            decode_step()

    # Untimed: bring the GPU to its steady clocks first (the first few hundred launches after the
    # host-side set-up run 5-10 % slower), then the W warm-up steps the caller asked for.
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_seconds:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: exactly K steps, queued back to back, nothing else on the stream; one HIP event on
    # the launch stream before the first step and one after the last give the region's duration on the GPU
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    region_us = ev0.elapsed_time(ev1) * 1e3 / args.steps
    # a second pass of K steps with events around the attention call, for the kernel's own duration
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in ev:
        if fused:
            a.record()
            fused_step()
            b.record()
        else:
            store_step()
            a.record()
            decode_step()
            b.record()
    torch.cuda.synchronize()
    dec_us = np.array([a.elapsed_time(b) for a, b in ev]) * 1e3
    dec_mean_us = float(dec_us.mean())

    progress(f"timed region done: {ms_per_step * 1e3:.2f} us per step (wall), {region_us:.2f} us (bracketing events), "
             f"{dec_mean_us:.2f} us per call (events around each call)")
    dbytes = decode_bytes(w, lens1)
    sbytes = store_bytes(w, B)
    value = (dbytes + sbytes) / (ms_per_step * 1e-3) / 1e9
    kernel_bytes = dbytes + (sbytes if fused else 0)          # the fused kernel also moves the new tokens
    # The dominant kernel's average launch duration.  With the fused step the timed region is K launches of
    # that one kernel and nothing else, so the events that bracket the region give it (including the gap
    # between two launches, a good microsecond); events recorded around every single call cost two more
    # records per launch and read 1-3 us higher: they are kept for the spread (median, p10, p90).
    launch_us = region_us if fused else dec_mean_us
    achieved = kernel_bytes / (launch_us * 1e-6) / 1e9

    result = {
        "metric": "INT4 paged decode attn HBM GB/s (% peak) + rotate-quant-store tokens/s",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {B}, context U[512,4096] (mean {w.seq_lens.mean():.0f}), "
                               f"{w.n_q_heads}q/{w.n_kv_heads}kv heads, head_dim {w.head_dim}, page 16, "
                               f"Hadamard block {w.had_block}, bf16 K/V with Student-t(3) channel scales",
                   "tokens_cached": int(lens1.sum()), "splits": splits, "chunk_tokens": chunk,
                   "bytes_per_step": dbytes + sbytes,
                   "call": ("saw_append_decode_attn" if order is None else "saw_append_decode_attn_hinted (the caller hands over the "
                            "longest-first order of the batch, computed once per decode step - i.e. once for all layers - by "
                            "saw_decode_order, outside the timed per-layer step: extra.decode_order_us; "
                            "extra.without_order_hint has the same step with the kernel ranking the sequences itself)")
                           if fused else "saw_rotate_quant_store + saw_paged_decode_attn"},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm",
                     "kernel": ("the step's call = one launch of decode_int4_mfma_kernel (pair mode, fused append)"
                                if fused else "saw_paged_decode_attn (decode_int4_mfma_kernel [+ merge])"),
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": profiled_traffic() if args.workload == "highconc" else None,
                     "bytes_per_launch": kernel_bytes, "avg_us": round(launch_us, 2),
                     "avg_us_from": ("two HIP events on the launch stream bracketing the K timed launches" if fused
                                     else "HIP events around every attention call"),
                     "per_call_events_us": {"avg": round(dec_mean_us, 2), "median": round(float(np.median(dec_us)), 2),
                                            "p10": round(float(np.percentile(dec_us, 10)), 2),
                                            "p90": round(float(np.percentile(dec_us, 90)), 2)}},
    }

    if extras:
        ex = {}
        med, mean, p10, p90 = time_calls(store_step, 50, 5)
        ex["decode_step_store_us"] = round(med, 2)
        med_d, mean, p10, p90 = time_calls(decode_step, 50, 5)
        ex["decode_only_us"] = round(med_d, 2)
        def wall_ms(fn, n=100):
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            t_a = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t_a) * 1e3 / n

        def unfused_step():
            store_step()
            decode_step()

        # same protocol for both (no events inside the loop): one call per step against two
        ex["unfused_step_ms"] = round(wall_ms(unfused_step), 5)
        ex["fused_step_ms"] = round(wall_ms(fused_step), 5)
        if order is not None:
            ex["decode_order_us"] = round(time_calls(lambda: saw.decode_order(seq_lens0, max_len0), 50, 5)[0], 2)
            # the same calls without the caller's order: every block ranks the 256 lengths itself first
            a, b = time_interleaved([lambda: saw.append_decode_attn(cache, newK, newV, q, pt, seq_lens0, max_seq_len=max_len0,
                                                                    out=out, workspace=ws),
                                     lambda: saw.paged_decode_attn(cache, q, pt, seq_lens, max_seq_len=max_len, out=out,
                                                                   workspace=ws, num_splits=args.num_splits)], 50, 5)
            ex["without_order_hint"] = {"fused_step_us": round(a, 2), "decode_only_us": round(b, 2),
                                        "fused_step_GB_s": round(kernel_bytes / a / 1e3, 1),
                                        "fused_step_pct_of_hbm_peak": round(kernel_bytes / a / 1e3 / HBM_PEAK_GBS * 100, 2)}
        ws16 = torch.empty(saw.decode_workspace_bytes(cache, B, w.n_q_heads, max_len), dtype=torch.uint8, device=dev)
        med, mean, p10, p90 = time_calls(lambda: saw.kv16_paged_decode_attn(kv16, q, pt, seq_lens, max_seq_len=max_len,
                                                                            out=out, workspace=ws16), 30, 5)
        b16 = kv16_decode_bytes(w, lens1)
        ex["kv16_decode"] = {"us": round(med, 2), "GB_s": round(b16 / med / 1e3, 1),
                             "pct_of_hbm_peak": round(b16 / med / 1e3 / HBM_PEAK_GBS * 100, 2),
                             # (against the INT4 decode that ranks the batch itself, as the 16-bit kernel does)
                             "int4_speedup": round(med / (ex["without_order_hint"]["decode_only_us"] if order is not None else med_d), 3),
                             "bytes_ratio": round(b16 / dbytes, 3),
                             "note": "16-bit baseline = MFMA kernel of the same design (direct K operand loads, "
                                     "HBM->LDS V tiles, LDS transpose reads, the same pair balancing of the ragged "
                                     "batch); at equal bandwidth the speed-up would equal bytes_ratio"}
        del kv16, ws16
        torch.cuda.empty_cache()
        progress("step variants and 16-bit baseline done")
        # what this machine's memory system delivers to a kernel that only reads, in the decode kernel's pattern
        rc = read_ceiling(saw, dev, w, cache)
        rc["decode_pct_of_read_ceiling"] = round(achieved / rc["decode_pattern"]["GB_s"] * 100, 2)
        rc["decode_only_pct_of_read_ceiling"] = round(dbytes / med_d / 1e3 / rc["decode_pattern"]["GB_s"] * 100, 2)
        ex["box_read_ceiling"] = rc
        # K-only rotation (the serving default of App. D): V is stored as plain INT4 and the output is not rotated back
        ck = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, 1, device=dev)
        fill(w, saw, dev, ck)
        kd, kf = time_interleaved([lambda: saw.paged_decode_attn(ck, q, pt, seq_lens, max_seq_len=max_len, out=out, workspace=ws),
                                   lambda: saw.append_decode_attn(ck, newK, newV, q, pt, seq_lens0, max_seq_len=max_len0, out=out, workspace=ws)],
                                  50, 5)
        ex["k_only_rotation"] = {"decode_only_us": round(kd, 2), "fused_step_us": round(kf, 2),
                                 "decode_only_vs_k_and_v": round(kd / med_d, 4)}
        del ck
        torch.cuda.empty_cache()
        # learned per-layer rotation after the Hadamard (App. A.3; a seeded random orthogonal matrix stands in for it):
        # the query, the appended token and the output take one more 128 x 128 product each
        cl = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask, device=dev,
                       dense=synth.random_orthogonal(w.head_dim, 2))
        fill(w, saw, dev, cl)
        ld_, lf_ = time_interleaved([lambda: saw.paged_decode_attn(cl, q, pt, seq_lens, max_seq_len=max_len, out=out, workspace=ws,
                                                                   order=order),
                                     lambda: saw.append_decode_attn(cl, newK, newV, q, pt, seq_lens0, max_seq_len=max_len0, out=out,
                                                                    workspace=ws, order=order)], 50, 5)
        ex["learned_rotation"] = {"decode_only_us": round(ld_, 2), "fused_step_us": round(lf_, 2),
                                  "decode_only_vs_hadamard_only": round(ld_ / med_d, 4)}
        del cl
        torch.cuda.empty_cache()
        progress("read ceiling and K-only done")
        ex["prefill_store_sweep"] = store_sweep(saw, dev)
        progress("store sweep done")
        ex["prefill_flatten_sweep"] = flatten_sweep(saw, dev)
        progress("flatten sweep done")
        del cache
        torch.cuda.empty_cache()
        ceiling = copy_ceiling(dev)
        ex["box_copy_ceiling"] = {"GB_s": round(ceiling, 1), "pct_of_hbm_peak": round(ceiling / HBM_PEAK_GBS * 100, 2),
                                  "decode_pct_of_ceiling": round(achieved / ceiling * 100, 2),
                                  "what": "1 GiB device-to-device copy, read + written bytes per second"}
        w2 = synth.make_workload("llama8b")
        c2 = saw.Cache(w2.num_pages, w2.n_kv_heads, w2.head_dim, w2.had_block, w2.rotate_mask, device=dev)
        K2 = torch.cat([synth.gen_kv(w2, b, 4096, 4097, device=dev)[0] for b in range(w2.batch)])
        V2 = torch.cat([synth.gen_kv(w2, b, 4096, 4097, device=dev)[1] for b in range(w2.batch)])
        pt2 = torch.from_numpy(w2.page_table).to(dev)
        sl2 = torch.from_numpy(np.stack([np.arange(w2.batch, dtype=np.int32), np.full(w2.batch, 4096, np.int32)], 1)).to(dev)
        med, mean, p10, p90 = time_calls(lambda: saw.rotate_quant_store(c2, K2, V2, pt2, sl2), 50, 5)
        ex["llama8b_store_16_new_tokens_us"] = round(med, 2)          # launch-latency dominated
        del c2
        ex["llama8b_store_32_layers"] = layers_store(saw, dev)
        progress("store latencies done")
        ex["other_decode"] = {
            # equal lengths: neither kernel needs balancing, so the 16-bit comparison isolates the format
            "highconc_uniform2304": other_decode(saw, dev, "highconc", ctx=2304, with_kv16=True),
            "llama8b": other_decode(saw, dev, "llama8b", with_append=True),
            "longctx1": other_decode(saw, dev, "longctx1"),
            "longctx4": other_decode(saw, dev, "longctx4"),
            # 1024 (sequence, kv head) items: pair blocks of four wavefronts
            "highconc_4kv_heads": other_decode(saw, dev, "highconc", n_q_heads=16, n_kv_heads=4),
            # head_dim 64 (two kv heads per block as one 128-channel row), Llama-3.2-1B-like heads
            "highconc_head_dim64": other_decode(saw, dev, "highconc", head_dim=64, had_block=64, with_append=True),
            # mid-size ragged batch (384 items: partitions + merge) and equal lengths just above 2048 items
            "highconc_48_sequences": other_decode(saw, dev, "highconc", batch=48),
            # small batch of short contexts: one block of eight wavefronts per (sequence, kv head), one launch
            "small_32x2304": other_decode(saw, dev, "llama8b", batch=32, ctx=2304, with_append=True),
            "small_4x2304": other_decode(saw, dev, "llama8b", batch=4, ctx=2304, with_append=True),
            "highconc_260_equal2304": other_decode(saw, dev, "highconc", batch=260, ctx=2304),
        }
        u = ex["other_decode"]["highconc_uniform2304"]["kv16_decode"]
        ex["int4_vs_16bit_decode"] = {
            "ragged_speedup": ex["kv16_decode"]["int4_speedup"],     # both kernels balance the ragged batch the same way
            "equal_lengths_speedup": u["int4_speedup"],
            "bytes_ratio": u["bytes_ratio"]}
        result["extra"] = ex

    progress("GPU part done")
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
