"""qesgd_round (a whole round in one call; one launch where the shape allows it) against the
two-call form qesgd_quantize_pack_batched + qesgd_unpack_aggregate_update and against the oracle:
packed blocks, zbar, u and zsum bit for bit."""
import numpy as np
import pytest
import torch

from test_gpu_parity import B, S  # noqa: F401

pytestmark = pytest.mark.gpu


def both_forms(B, slab, center, d, s, bucket, norm_kind, seed, rnd, K, w, zsum0, with_zbar=True, with_zsum=True):
    lay = B.qesgd_layout_query(d, s, bucket)
    wsb = B.qesgd_workspace_bytes(d, s, bucket, K)
    ws = torch.empty(max(wsb, 4) // 4, device="cuda") if wsb else None
    out = []
    for fused in (False, True):
        packed = B.alloc_packed(lay, K)
        packed.fill_(0xA5)
        zbar = torch.full((d,), float("nan"), device="cuda") if with_zbar else None
        u = torch.full((d,), float("nan"), device="cuda")
        zsum = zsum0.clone() if with_zsum else None
        if fused:
            B.qesgd_round(slab, slab.stride(0) if K > 1 else 0, center, d, s, bucket, norm_kind, seed, rnd, K, packed,
                          packed.stride(0), w, zbar, u, zsum, workspace=ws)
        else:
            B.qesgd_quantize_pack_batched(slab, slab.stride(0) if K > 1 else 0, center, d, s, bucket, norm_kind, seed,
                                          rnd, K, packed, packed.stride(0), ws)
            B.qesgd_unpack_aggregate_update(packed, packed.stride(0), K, d, s, bucket, w, zbar, u, zsum)
        torch.cuda.synchronize()
        out.append((packed, zbar, u, zsum))
    return lay, out


def assert_same(out):
    (p0, z0, u0, s0), (p1, z1, u1, s1) = out
    assert torch.equal(p0, p1), "packed blocks differ"
    assert torch.equal(u0.view(torch.int32), u1.view(torch.int32)), "u differs"
    if z0 is not None:
        assert torch.equal(z0.view(torch.int32), z1.view(torch.int32)), "zbar differs"
    if s0 is not None:
        assert torch.equal(s0.view(torch.int32), s1.view(torch.int32)), "zsum differs"


def make_inputs(d, K, seed, with_center):
    g = torch.Generator(device="cpu").manual_seed(seed)
    stride = (d + 63) // 64 * 64
    slab = torch.zeros(max(K, 1), stride)
    c = torch.randn(d, generator=g) if with_center else None
    slab[:, :d] = torch.randn(K, d, generator=g) * 1e-3 * (1 + torch.arange(K))[:, None]
    if with_center:
        slab[:, :d] += c[None, :]
    w = torch.randn(d, generator=g)
    zsum0 = torch.randn(d, generator=g) * 1e-2
    return slab.cuda(), (None if c is None else c.cuda()), w.cuda(), zsum0.cuda()


@pytest.mark.parametrize("log2n", range(5, 16))
@pytest.mark.parametrize("s,K", [(2, 8), (4, 3), (16, 1), (256, 5), (65536, 2)])
def test_one_launch_shapes_equal_two_calls(B, log2n, s, K):
    bucket = 1 << log2n
    tile = max(4096, bucket) * (4 if log2n == 15 else 1)
    for d in (2 * tile, tile + bucket + 37, 1000):            # whole tiles; tiles + ragged tail; less than a tile
        slab, _, w, zsum0 = make_inputs(d, K, log2n * 7 + s, False)
        _, out = both_forms(B, slab, None, d, s, bucket, 0, 99, log2n, K, w, zsum0)
        assert_same(out)


@pytest.mark.parametrize("d,bucket,s,K", [(4096 * 5 + 100, 512, 16, 4), (8192 * 3 + 8, 8192, 256, 3), (70_001, 4096, 2, 16)])
def test_center_and_optional_outputs(B, d, bucket, s, K):
    slab, c, w, zsum0 = make_inputs(d, K, d, True)
    _, out = both_forms(B, slab, c, d, s, bucket, 0, 5, 1, K, w, zsum0)
    assert_same(out)
    _, out = both_forms(B, slab, c, d, s, bucket, 0, 5, 2, K, w, zsum0, with_zbar=False, with_zsum=False)
    assert_same(out)


@pytest.mark.parametrize("d,bucket,s,K,norm_kind", [
    (50_000, 96, 16, 3, 0),          # bucket not a power of two
    (50_000, 512, 16, 3, 1),         # max norm
    (50_000, 512, 8, 3, 0),          # level width that does not divide a word
    (150_000, 65_536, 4, 3, 0),      # wide bucket (needs the workspace)
    (9_000, 1 << 20, 4, 2, 0)])      # one bucket, not a power of two
def test_other_shapes_fall_back_to_two_launches(B, d, bucket, s, K, norm_kind):
    slab, _, w, zsum0 = make_inputs(d, K, d + s, False)
    _, out = both_forms(B, slab, None, d, s, bucket, norm_kind, 7, 3, K, w, zsum0)
    assert_same(out)


@pytest.mark.parametrize("name,d", [("cfg1", 16_384), ("cfg2", 1_048_576), ("cfg3", 41_034), ("cfg4", 70_008),
                                    ("cfg5", 61_000)])
def test_round_matches_oracle(oracle, B, S, name, d):
    cfg = S.by_name(name).scaled(d=d, K=min(S.by_name(name).K, 4))
    slab = S.worker_slab(cfg, "cuda")
    w = S.snapshot(cfg, "cuda")
    lay = B.qesgd_layout_query(cfg.d, cfg.s, cfg.bucket)
    packed = B.alloc_packed(lay, cfg.K)
    zbar = torch.empty(cfg.d, device="cuda")
    u = torch.empty(cfg.d, device="cuda")
    zsum = torch.zeros(cfg.d, device="cuda")
    host = slab[:, :cfg.d].cpu().numpy()
    ozsum = np.zeros(cfg.d, np.float32)
    for rnd in range(2):
        B.qesgd_round(slab, slab.stride(0), None, cfg.d, cfg.s, cfg.bucket, 0, cfg.seed, rnd, cfg.K, packed,
                      packed.stride(0), w, zbar, u, zsum)
        torch.cuda.synchronize()
        planes = [oracle.quantize_pack(host[k], cfg.s, cfg.bucket, cfg.seed, rnd, k) for k in range(cfg.K)]
        for k in range(cfg.K):
            n, sg, lv = B.planes(packed[k], lay)
            assert np.array_equal(n.cpu().numpy().view(np.uint32), planes[k][0].view(np.uint32))
            assert np.array_equal(sg.cpu().numpy().view(np.uint32), planes[k][1])
            assert np.array_equal(lv.cpu().numpy().view(np.uint32), planes[k][2])
        oz = oracle.unpack_aggregate(np.stack([p[0] for p in planes]), np.stack([p[1] for p in planes]),
                                     np.stack([p[2] for p in planes]), cfg.d, cfg.s, cfg.bucket)
        ou, ozsum = oracle.apply_update(w.cpu().numpy(), oz, ozsum)
        for got, want in ((zbar, oz), (u, ou), (zsum, ozsum)):
            assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_round_argument_errors(B):
    L = B.lib()
    x, pk, w, z, u = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
    f = L.qesgd_round
    assert f(None, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_NULL
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, None, z, u, None, None) == B.ERR_NULL
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, None, None, None) == B.ERR_NULL
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 0, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_WORKERS
    assert f(x, 4096, None, 4096, 3, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_LEVELS
    assert f(x, 100_000, None, 100_000, 4, 100_000, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u, None, None) == B.ERR_WORKSPACE
    assert f(x, 4096, None, 4096, 4, 512, 0, 1, 0, 2, pk, 1 << 20, None, 0, w, z, u + 4, None, None) == B.ERR_ALIGN
