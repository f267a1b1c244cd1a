"""Whole-output parity at the five full sizes, in the launch configuration the benchmark times.

For every configuration, every round it names and every worker: all bucket scales, all sign words
and all level words of qesgd_quantize_pack_batched against the oracle's quantize_pack, bit for bit;
then qesgd_unpack_aggregate_update on the quantiser's own packed output against the oracle's
unpack_aggregate + apply_update on the oracle's own planes, every coordinate of zbar, u and zsum
(bit for bit, which also meets the 1e-6 bar), with zsum carried from round to round.  In round r
worker k quantises pool vector (k + r) mod K with the variates of (seed, round r, worker k).

The oracle is single-threaded; its K per-worker calls and the ranges of the aggregate run on host
threads (ctypes releases the interpreter lock), so the largest configuration costs a few seconds
per round.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from test_gpu_parity import B, S, rel_err  # noqa: F401

pytestmark = pytest.mark.gpu

THREADS = max(1, min(16, os.cpu_count() or 1))


def oracle_round(oracle, pool, host, order, cfg, rnd, w_host, zsum_host):
    """One round on the CPU: -> (planes per worker, zbar, u, zsum)."""
    d, K, s, bucket = cfg.d, cfg.K, cfg.s, cfg.bucket
    planes = list(pool.map(lambda k: oracle.quantize_pack(host[order[k]], s, bucket, cfg.seed, rnd, k), range(K)))
    norms = np.stack([p[0] for p in planes])
    sw = np.stack([p[1] for p in planes])
    lw = np.stack([p[2] for p in planes])
    Bk = min(bucket, d)
    per = max(Bk, (d // THREADS + Bk) // Bk * Bk)            # bucket-aligned ranges, one per thread
    cuts = list(range(0, d, per)) + [d]

    def part(j):
        a, e = cuts[j], cuts[j + 1]
        z = oracle.unpack_aggregate(norms, sw, lw, d, s, bucket, a, e)
        u, zs = oracle.apply_update(w_host[a:e], z, zsum_host[a:e])
        return z, u, zs

    parts = list(pool.map(part, range(len(cuts) - 1)))
    zbar = np.concatenate([p[0] for p in parts])
    u = np.concatenate([p[1] for p in parts])
    zsum = np.concatenate([p[2] for p in parts])
    return planes, zbar, u, zsum


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_every_bit_of_every_round(oracle, B, S, name):
    cfg = S.by_name(name)
    d, K, s, bucket = cfg.d, cfg.K, cfg.s, cfg.bucket
    slab = S.worker_slab(cfg, "cuda")
    w = S.snapshot(cfg, "cuda")
    host = slab[:, :d].cpu().numpy()
    w_host = w.cpu().numpy()
    assert np.isfinite(host).all()
    lay = B.qesgd_layout_query(d, s, bucket)
    packed = B.alloc_packed(lay, K)
    rot = torch.empty_like(slab) if cfg.rounds > 1 else slab
    zbar = torch.empty(d, device="cuda")
    u = torch.empty(d, device="cuda")
    zsum = torch.zeros(d, device="cuda")
    ozsum = np.zeros(d, np.float32)
    with ThreadPoolExecutor(max_workers=THREADS) as pool:
        for rnd in range(cfg.rounds):
            print(f"{name} round {rnd} of {cfg.rounds}: d={d} K={K} s={s} bucket={bucket}", flush=True)
            order = [(k + rnd) % K for k in range(K)]
            if cfg.rounds > 1:
                for k in range(K):
                    rot[k].copy_(slab[order[k]])
            packed.fill_(0xA5)
            B.qesgd_quantize_pack_batched(rot, rot.stride(0), None, d, s, bucket, B.NORM_L2, cfg.seed, rnd, K,
                                          packed, packed.stride(0))
            B.qesgd_unpack_aggregate_update(packed, packed.stride(0), K, d, s, bucket, w, zbar, u, zsum)
            torch.cuda.synchronize()
            planes, oz, ou, ozsum = oracle_round(oracle, pool, host, order, cfg, rnd, w_host, ozsum)
            for k in range(K):
                n, sg, lv = B.planes(packed[k], lay)
                got_n = n.cpu().numpy().view(np.uint32)
                bad = np.nonzero(got_n != planes[k][0].view(np.uint32))[0]
                assert bad.size == 0, f"round {rnd} worker {k}: {bad.size} bucket scales differ, first {bad[:5]}"
                got_s = sg.cpu().numpy().view(np.uint32)
                bad = np.nonzero(got_s != planes[k][1])[0]
                assert bad.size == 0, f"round {rnd} worker {k}: {bad.size} sign words differ, first {bad[:5]}"
                got_l = lv.cpu().numpy().view(np.uint32)
                bad = np.nonzero(got_l != planes[k][2])[0]
                assert bad.size == 0, f"round {rnd} worker {k}: {bad.size} level words differ, first {bad[:5]}"
            for got, want, what in ((zbar, oz, "zbar"), (u, ou, "u"), (zsum, ozsum, "zsum")):
                g = got.cpu().numpy()
                assert rel_err(g, want) <= 1e-6, (rnd, what)
                bad = np.nonzero(g.view(np.uint32) != want.view(np.uint32))[0]
                assert bad.size == 0, f"round {rnd}: {bad.size} coordinates of {what} differ, first {bad[:5]}"
