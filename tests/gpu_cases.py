"""Shared drivers for the GPU parity tests: run a synthetic workload through the HIP path and
through the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import parity
from oracle import saw_oracle as O
from paper_2604_19157_amd import synth


def fill_caches(w, saw, dev="cuda", chunk=4096, order_rng=None, with_ref=True):
    """Store every token of every sequence of `w`; returns (gpu cache, oracle cache, per-vector records)."""
    cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask, device=dev, signs=w.signs, dense=w.dense)
    ref = O.new_cache(w.num_pages, w.n_kv_heads, w.page_size, w.head_dim) if with_ref else None
    pt = torch.from_numpy(w.page_table).to(dev)
    recs = []
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        for p0 in range(0, L, chunk):
            p1 = min(L, p0 + chunk)
            K, V = synth.gen_kv(w, b, p0, p1)
            sl = synth.slots_for(b, p0, p1)
            if order_rng is not None:                      # tokens of a call in arbitrary order
                perm = order_rng.permutation(p1 - p0)
                K, V, sl = K[perm].contiguous(), V[perm].contiguous(), sl[perm]
            saw.rotate_quant_store(cache, K.to(dev), V.to(dev), pt, torch.from_numpy(sl).to(dev))
            if with_ref:
                r = O.rotate_quant_store(ref, K.float().numpy(), V.float().numpy(), w.page_table, sl,
                                         w.had_block, w.rotate_mask, return_prerounding=True, signs=w.signs, dense=w.dense)
                recs.append(r)
    torch.cuda.synchronize()
    return cache, ref, recs, pt


def oracle_fill(w, chunk=4096, seqs=None):
    """The oracle's cache for `w` (all sequences, or only `seqs`), written by the oracle's own store."""
    ref = O.new_cache(w.num_pages, w.n_kv_heads, w.page_size, w.head_dim)
    for b in (range(w.batch) if seqs is None else seqs):
        L = int(w.seq_lens[b])
        for p0 in range(0, L, chunk):
            p1 = min(L, p0 + chunk)
            K, V = synth.gen_kv(w, b, p0, p1)
            O.rotate_quant_store(ref, K.float().numpy(), V.float().numpy(), w.page_table,
                                 synth.slots_for(b, p0, p1), w.had_block, w.rotate_mask, signs=w.signs, dense=w.dense)
    return ref


def upload_cache(ref, w, saw, dev="cuda", into=None, pages=None):
    """Copy an oracle cache's bytes into a device cache (a new one, or rows `pages` of `into`)."""
    cache = into if into is not None else saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block,
                                                    w.rotate_mask, device=dev, signs=w.signs, dense=w.dense)
    for k in ("k_codes", "v_codes", "k_meta", "v_meta"):
        dst = getattr(cache, k)
        if pages is None:
            dst.copy_(torch.from_numpy(ref[k]).reshape(dst.shape))
        else:
            idx = torch.from_numpy(np.asarray(pages, np.int64)).to(dev)
            src = torch.from_numpy(ref[k][np.asarray(pages)]).to(dev)
            dst.view(dst.shape[0], -1)[idx] = src.reshape(len(pages), -1).to(dst.dtype)
    torch.cuda.synchronize()
    return cache


def cache_to_numpy(cache, w):
    d = {k: getattr(cache, k).cpu().numpy() for k in ("k_codes", "v_codes", "k_meta", "v_meta")}
    d.update(page_size=w.page_size, head_dim=w.head_dim, n_kv_heads=w.n_kv_heads)
    return d


def compare_store(got: dict, ref: dict, recs: list) -> dict:
    """Classify every stored vector (see parity.compare_vectors) and check nothing else was written."""
    total = None
    written = np.zeros(ref["k_codes"].shape[:3], bool)
    for r in recs:
        page, slot = r["page"], r["slot"]
        written[page, :, slot] = True
        for which in ("k", "v"):
            cg = got[which + "_codes"][page, :, slot, :]
            cr = ref[which + "_codes"][page, :, slot, :]
            mg = got[which + "_meta"][page, :, slot, :]
            mr = ref[which + "_meta"][page, :, slot, :]
            n = cg.shape[0] * cg.shape[1]
            d = r[which + "_y"].shape[-1]
            res = parity.compare_vectors(cg.reshape(n, -1), mg.reshape(n, 2), cr.reshape(n, -1), mr.reshape(n, 2),
                                         r[which + "_y"].reshape(n, d), r[which + "_s"].reshape(n),
                                         r[which + "_z"].reshape(n))
            if total is None:
                total = res
            else:
                for k, v in res.items():
                    if k == "scale_max_rel":
                        total[k] = max(total[k], v)
                    elif k == "first_hard":
                        total[k] = (total[k] + v)[:5]
                    else:
                        total[k] += v
    untouched_ok = True
    for which in ("k", "v"):
        untouched_ok &= not got[which + "_codes"][~written].any()
        untouched_ok &= not got[which + "_meta"][~written].any()
    total["untouched_ok"] = bool(untouched_ok)
    return total
