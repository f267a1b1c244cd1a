"""Whole-output checks at the five full sizes, in the launch configuration the benchmark times.

The element-by-element comparison with the oracle covers sampled buckets at these sizes; here
every coordinate of a worker's packed output is decoded with plain torch integer ops and checked
against what Eq. (2) of Sec. 2.1 fixes for any input:
  * every level lies in [0, s-1] and the unused high bits of both planes are 0;
  * the decoded value is one of the two grid neighbours of the input: |Q(v)_i - v_i| <= step_b;
  * values on the grid (here: exact zeros) do not move;
  * the bucket scales equal the L2 norms computed in fp64 within 1e-6;
  * the rounding is unbiased: the mean of (Q(v)_i - v_i)/step_b over all coordinates is zero
    within four standard errors (variance <= 1/4 per coordinate, Lemma 1) plus the 2^-16 bias
    of the 16-bit variate.
"""
import math

import pytest
import torch

from test_gpu_parity import B, S  # noqa: F401

pytestmark = pytest.mark.gpu


def decode_plane(words_i32, d, bits):
    """[n_words] int32 -> [d] int32 fields of `bits` bits each (bits divides 32)."""
    per = 32 // bits
    shifts = torch.arange(per, device=words_i32.device, dtype=torch.int32) * bits
    fields = (words_i32[:, None] >> shifts[None, :]) & ((1 << bits) - 1)
    return fields.reshape(-1)[:d]


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_every_coordinate_of_a_worker(B, S, name):
    cfg = S.by_name(name)
    d, K, s, bucket = cfg.d, cfg.K, cfg.s, cfg.bucket
    slab = S.worker_slab(cfg, "cuda")
    lay = B.qesgd_layout_query(d, s, bucket)
    m = lay.level_bits
    packed = B.alloc_packed(lay, K)
    packed.zero_()
    B.qesgd_quantize_pack_batched(slab, slab.stride(0), None, d, s, bucket, 0, cfg.seed, 2, K, packed,
                                  packed.stride(0))
    torch.cuda.synchronize()
    Bk = min(bucket, d)
    nb = lay.n_buckets
    for k in sorted({0, K - 1}):
        v = slab[k, :d]
        norms, sg, lv = B.planes(packed[k], lay)
        sign = decode_plane(sg.view(torch.int32), d, 1)
        level = decode_plane(lv.view(torch.int32), d, m)
        assert int(level.max()) <= s - 1 and int(level.min()) >= 0
        if d % 32:
            assert (int(sg.view(torch.int32)[-1].item()) & 0xFFFFFFFF) >> (d % 32) == 0
        used = (d * m) % 32
        if used:
            assert (int(lv.view(torch.int32)[-1].item()) & 0xFFFFFFFF) >> used == 0
        # bucket scales against fp64
        pad = nb * Bk - d
        v64 = torch.nn.functional.pad(v.double(), (0, pad)).view(nb, Bk)
        ref = v64.pow(2).sum(dim=1).sqrt()
        rel = ((norms.double() - ref).abs() / ref.clamp_min(1e-300)).max()
        assert float(rel) <= 1e-6, float(rel)
        del v64
        step = (norms / float(s - 1)).repeat_interleave(Bk)[:d]
        q = level.float() * step
        q = torch.where(sign == 1, -q, q)
        err = (q - v).abs()
        # one grid step, plus the rounding of inv = fl((s-1)/norm) against step = fl(norm/(s-1)) at a <= s-1
        assert bool((err <= step * (1.0 + 4e-7 * s)).all()), float((err / step.clamp_min(1e-30)).max())
        assert bool((sign == (v < 0).int()).all())
        zeros = v == 0
        if bool(zeros.any()):
            assert bool((level[zeros] == 0).all())
        live = step > 0
        t = ((q - v)[live].double() / step[live].double())
        n = int(live.sum())
        assert abs(float(t.mean())) <= 4 * 0.5 / math.sqrt(n) + 2.0 ** -16, (float(t.mean()), n)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_aggregate_every_coordinate_against_fp64(B, S, name):
    """zbar at full size against the sum over workers recomputed in fp64 from planes decoded with
    torch integer ops (Alg. 3, server task): |zbar - mean| <= (K+3) 2^-24 mean|q| for every
    coordinate; u and zsum are then exact fp32 sums of their inputs."""
    from test_gpu_parity import random_packed
    cfg = S.by_name(name)
    d, K, s, bucket = cfg.d, cfg.K, cfg.s, cfg.bucket
    lay, packed = random_packed(B, S, d, s, bucket, K, seed=cfg.seed + 100)
    m = lay.level_bits
    Bk = min(bucket, d)
    w = S.snapshot(cfg, "cuda")
    zsum0 = torch.empty(d, device="cuda").normal_(0.0, 1e-3, generator=torch.Generator(device="cuda").manual_seed(3))
    zsum = zsum0.clone()
    zbar = torch.empty(d, device="cuda")
    u = torch.empty(d, device="cuda")
    B.qesgd_unpack_aggregate_update(packed, packed.stride(0), K, d, s, bucket, w, zbar, u, zsum)
    torch.cuda.synchronize()
    total = torch.zeros(d, dtype=torch.float64, device="cuda")
    mag = torch.zeros(d, dtype=torch.float64, device="cuda")
    for k in range(K):
        norms, sg, lv = B.planes(packed[k], lay)
        sign = decode_plane(sg, d, 1)
        level = decode_plane(lv, d, m)
        q = level.double() * (norms.double() / float(s - 1)).repeat_interleave(Bk)[:d]
        mag += q
        total += torch.where(sign == 1, -q, q)
        del sign, level, q
    want = total / K
    bound = (K + 3) * 2.0 ** -24 * mag / K + 1e-45
    assert bool(((zbar.double() - want).abs() <= bound).all())
    assert torch.equal(u, w + zbar) and torch.equal(zsum, zsum0 + zbar)
