"""More shapes through the specialised quantize kernel: every power-of-two bucket from 32 to 32768,
every level width, vectors that are an exact multiple of the tile, smaller than a tile, and one
coordinate longer; 64 workers in one launch."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1901_03040_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


def run_and_compare(oracle, B, x, s, bucket, seed, rnd, K=1, center=None, d=None):
    d = x.shape[-1] if d is None else d
    lay = B.qesgd_layout_query(d, s, bucket)
    packed = B.alloc_packed(lay, K)
    packed.fill_(0xA5)
    if K == 1:
        B.qesgd_quantize_pack(x, center, d, s, bucket, 0, seed, rnd, 0, packed)
    else:
        B.qesgd_quantize_pack_batched(x, x.stride(0), center, d, s, bucket, 0, seed, rnd, K, packed, packed.stride(0))
    torch.cuda.synchronize()
    xh = x.cpu().numpy().reshape(K, -1)
    ch = None if center is None else center.cpu().numpy()
    assert np.isfinite(xh).all() and (ch is None or np.isfinite(ch).all()), "inputs changed on the device"
    for k in range(K):
        n, sg, lv = B.planes(packed[k], lay)
        on, osw, olw = oracle.quantize_pack(xh[k, :d], s, bucket, seed, rnd, k, center=ch)
        assert np.array_equal(n.cpu().numpy().view(np.uint32), on.view(np.uint32)), (k, "norms")
        assert np.array_equal(sg.cpu().numpy().view(np.uint32), osw), (k, "signs")
        assert np.array_equal(lv.cpu().numpy().view(np.uint32), olw), (k, "levels")


@pytest.mark.parametrize("log2n", range(5, 16))
@pytest.mark.parametrize("s", [2, 4, 16, 256, 65536])
def test_every_power_of_two_bucket(oracle, B, log2n, s):
    bucket = 1 << log2n
    tile = max(4096, bucket)
    g = torch.Generator(device="cpu").manual_seed(log2n * 100 + s)
    for d in (3 * tile, 2 * tile + bucket + 37):          # whole tiles only; tiles + a ragged tail
        x = (torch.randn(d, generator=g) * 1e-2).cuda()
        run_and_compare(oracle, B, x, s, bucket, 99, log2n)


@pytest.mark.parametrize("d", [4095, 4096, 4097, 8191, 8192, 12288 + 8])
def test_around_one_tile(oracle, B, d):
    g = torch.Generator(device="cpu").manual_seed(d)
    x = (torch.randn(d, generator=g) * 1e-2).cuda()
    for bucket in (128, 4096):
        run_and_compare(oracle, B, x, 16, bucket, 5, 1)


def test_sixty_four_workers_with_center(oracle, B):
    d, K = 10_000, 64
    g = torch.Generator(device="cpu").manual_seed(1)
    stride = (d + 63) // 64 * 64
    slab = torch.zeros(K, stride)
    slab[:, :d] = torch.randn(K, d, generator=g) * 1e-3
    c = torch.randn(d, generator=g) * 1e-3
    run_and_compare(oracle, B, slab.cuda(), 4, 1024, 3, 9, K=K, center=c.cuda(), d=d)


@pytest.mark.parametrize("K", [1, 3, 8])
@pytest.mark.parametrize("d,bucket,s", [(4096 * 19 + 100, 512, 16), (8192 * 9 + 8, 8192, 256), (4096 * 8, 4096, 2),
                                        (4096 * 7 + 4000, 64, 4), (32768 * 8 + 5, 32768, 4)])
def test_batched_with_center_tile_order(oracle, B, K, d, bucket, s):
    """With a center the workgroups of a launch take (worker, tile) in an order of their own (the
    workers of one tile next to each other); every worker's output must not depend on it."""
    g = torch.Generator(device="cpu").manual_seed(d + K)
    stride = (d + 63) // 64 * 64
    slab = torch.zeros(K, stride)
    c = torch.randn(d, generator=g)
    slab[:, :d] = c[None, :] + torch.randn(K, d, generator=g) * 1e-3
    run_and_compare(oracle, B, slab.cuda() if K > 1 else slab[0, :d].contiguous().cuda(), s, bucket, 8, 2, K=K,
                    center=c.cuda(), d=d)


@pytest.mark.parametrize("d,bucket,s,K", [(4096 * 16400 + 77, 4096, 2, 2), (512 * 8 * 16390, 512, 16, 3)])
def test_center_form_with_many_tiles(oracle, B, d, bucket, s, K):
    """From 16384 tiles on, the center form lets one workgroup take a tile of every worker."""
    g = torch.Generator(device="cuda").manual_seed(d % 1000 + K)
    stride = (d + 63) // 64 * 64
    c = torch.randn(d, generator=g, device="cuda")
    slab = torch.zeros(K, stride, device="cuda")
    slab[:, :d] = c[None, :] + torch.randn(K, d, generator=g, device="cuda") * 1e-3
    run_and_compare(oracle, B, slab, s, bucket, 8, 2, K=K, center=c, d=d)


def test_bench_probe_kernels_stay_in_their_buffers():
    """The benchmark's plain streaming kernels (their own shared object, not part of the library):
    copy and update mix give the expected values, the packed mixes write exactly the stated sizes,
    and nothing beyond them is touched."""
    import bench
    probe = bench.load_probe()
    st = torch.cuda.current_stream()
    n = 3 * 4096
    g = torch.Generator(device="cuda").manual_seed(1)
    a = torch.randn(n + 64, generator=g, device="cuda")
    b = torch.randn(n + 64, generator=g, device="cuda")
    guard = 123.0
    c, d, e = (torch.full((n + 64,), guard, device="cuda") for _ in range(3))
    probe(bench.PROBE_UPDATE_MIX, a, b, c, d, e, n, st)
    torch.cuda.synchronize()
    assert torch.equal(c[:n], a[:n]) and torch.equal(e[:n], b[:n]) and torch.equal(d[:n], a[:n] + b[:n])
    assert all(bool((t[n:] == guard).all()) for t in (c, d, e))
    c.fill_(guard)
    probe(bench.PROBE_COPY, a, c, None, None, None, n, st)
    torch.cuda.synchronize()
    assert torch.equal(c[:n], a[:n]) and bool((c[n:] == guard).all())
    p0 = torch.full((n // 32 + 16,), guard, device="cuda")
    p1 = torch.full((n // 32 + 16,), guard, device="cuda")
    probe(bench.PROBE_QUANTIZE_MIX, a, p0, p1, None, None, n, st)
    codes = torch.full((n // 4 + 16,), guard, device="cuda")
    probe(bench.PROBE_BYTE_CODES_MIX, a, codes, None, None, None, n, st)
    before = b.clone()
    probe(bench.PROBE_READ, a, b, None, None, None, n, st)
    torch.cuda.synchronize()
    assert bool((p0[n // 32:] == guard).all()) and bool((p1[n // 32:] == guard).all())
    assert not bool((p0[:n // 32] == guard).any())
    assert bool((codes[n // 4:] == guard).all())
    assert torch.equal(b, before)
    with pytest.raises(RuntimeError):
        probe(7, a, b, None, None, None, n, st)
    with pytest.raises(RuntimeError):
        probe(bench.PROBE_COPY, a, b, None, None, None, n + 1, st)
