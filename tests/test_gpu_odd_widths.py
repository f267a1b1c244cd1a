"""Parity for the level counts whose field width does not divide a word (s = 8, 32, 64, 128:
3, 5, 6, 7 bits), where a coordinate's level can continue in the next word of the plane.

Same bar as the other parity tests: norms and code words bit-exact, fp32 outputs within 1e-6
(met bit for bit).  Sizes cover whole quads of lanes, a ragged last quad, buckets that are and
are not powers of two, a single bucket, the wide-bucket two-pass path, and vectors shorter than
one word.
"""
import numpy as np
import pytest
import torch

from test_gpu_parity import (B, S, TOL, assert_codes_equal, gpu_quantize, oracle_planes,  # noqa: F401
                             random_packed, rel_err)

pytestmark = pytest.mark.gpu

ODD = [8, 32, 64, 128]


@pytest.mark.parametrize("s", ODD)
@pytest.mark.parametrize("d,bucket", [
    (20_000, 512), (20_011, 2048), (33_001, 4096), (70_003, 32_768), (5_003, 64), (9_999, 96),
    (9_001, 1_000_000), (40_000, 40_000), (150_001, 65_536), (300_001, 131_072 * 2), (200_003, 48_000)])
def test_quantize_pack_matches_oracle(oracle, B, s, d, bucket):
    g = torch.Generator(device="cpu").manual_seed(d * 31 + s)
    x = (torch.randn(d, generator=g) * 1e-3).to(torch.float32)
    seed, rnd, worker = 0xBEEF0000 + s, 2, 7
    lay, packed = gpu_quantize(B, x.cuda(), s, bucket, seed, rnd, worker)
    assert_codes_equal(oracle, B, x.numpy(), s, bucket, seed, rnd, worker, lay, packed[0])


@pytest.mark.parametrize("s", ODD)
def test_tiny_and_ragged_sizes(oracle, B, s):
    for d in [1, 2, 7, 8, 9, 10, 11, 15, 16, 17, 24, 25, 31, 32, 33, 40, 63, 64, 65, 95, 97, 255, 511, 513, 4097]:
        g = torch.Generator(device="cpu").manual_seed(d)
        x = (torch.randn(d, generator=g) * 0.1).to(torch.float32)
        for bucket in {d, 32, 1 << 20}:
            lay, packed = gpu_quantize(B, x.cuda(), s, bucket, 11, 0, 0)
            assert_codes_equal(oracle, B, x.numpy(), s, bucket, 11, 0, 0, lay, packed[0])
            # words after the last one of the level plane keep the poison written before the call
            tail = packed[0, lay.levels_off + 4 * lay.level_words: lay.levels_off + 4 * lay.level_words + 64]
            assert bool((tail == 0xA5).all()), (d, bucket)


@pytest.mark.parametrize("s", ODD)
@pytest.mark.parametrize("norm_kind", [0, 1])
def test_center_and_max_norm(oracle, B, s, norm_kind):
    d, bucket = 50_001, 512
    g = torch.Generator(device="cpu").manual_seed(7)
    w = torch.randn(d, generator=g).to(torch.float32)
    x = w + (torch.randn(d, generator=g) * 1e-3).to(torch.float32)
    lay, packed = gpu_quantize(B, x.cuda(), s, bucket, 5, 1, 2, center=w.cuda(), norm_kind=norm_kind)
    assert_codes_equal(oracle, B, x.numpy(), s, bucket, 5, 1, 2, lay, packed[0], center_host=w.numpy(),
                       norm_kind=norm_kind)


@pytest.mark.parametrize("s,K", [(8, 5), (32, 8), (64, 3), (128, 16), (8, 64)])
@pytest.mark.parametrize("d,bucket", [(30_000, 512), (30_005, 4096), (9_999, 96), (1001, 5000), (7, 32), (33, 32)])
def test_unpack_aggregate_update_matches_oracle(oracle, B, S, s, K, d, bucket):
    lay, packed = random_packed(B, S, d, s, bucket, K, seed=s + K)
    g = torch.Generator(device="cpu").manual_seed(d)
    w = torch.randn(d, generator=g)
    zsum0 = torch.randn(d, generator=g) * 1e-2
    zbar = torch.full((d,), float("nan"), device="cuda")
    u = torch.full((d,), float("nan"), device="cuda")
    zsum = zsum0.cuda()
    B.qesgd_unpack_aggregate_update(packed, packed.stride(0), K, d, s, bucket, w.cuda(), zbar, u, zsum)
    torch.cuda.synchronize()
    norms, sw, lw = oracle_planes(B, packed, lay, K)
    ozbar = oracle.unpack_aggregate(norms, sw, lw, d, s, bucket)
    ou, ozsum = oracle.apply_update(w.numpy(), ozbar, zsum0.numpy())
    for got, want, what in [(zbar, ozbar, "zbar"), (u, ou, "u"), (zsum, ozsum, "zsum")]:
        got = got.cpu().numpy()
        assert rel_err(got, want) <= TOL, what
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{what} not bit-exact"


@pytest.mark.parametrize("s", ODD)
def test_full_round(oracle, B, S, s):
    """quantize -> aggregate -> update, each side on its own intermediates."""
    cfg = S.by_name("cfg3").scaled(d=41_034, K=4)
    slab = S.worker_slab(cfg, "cuda")
    w = S.snapshot(cfg, "cuda")
    host = slab[:, :cfg.d].cpu().numpy()
    lay = B.qesgd_layout_query(cfg.d, s, cfg.bucket)
    packed = B.alloc_packed(lay, cfg.K)
    u = torch.empty(cfg.d, device="cuda")
    B.qesgd_quantize_pack_batched(slab, slab.stride(0), None, cfg.d, s, cfg.bucket, 0, cfg.seed, 0, cfg.K,
                                  packed, packed.stride(0))
    B.qesgd_unpack_aggregate_update(packed, packed.stride(0), cfg.K, cfg.d, s, cfg.bucket, w, None, u, None)
    torch.cuda.synchronize()
    op = [oracle.quantize_pack(host[k], s, cfg.bucket, cfg.seed, 0, k) for k in range(cfg.K)]
    oz = oracle.unpack_aggregate(np.stack([p[0] for p in op]), np.stack([p[1] for p in op]),
                                 np.stack([p[2] for p in op]), cfg.d, s, cfg.bucket)
    ou, _ = oracle.apply_update(w.cpu().numpy(), oz, None)
    assert np.array_equal(u.cpu().numpy(), ou)
