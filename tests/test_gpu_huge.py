"""Vectors beyond 2^32 and 2^35 coordinates: 64-bit indexing in the kernels and the high word of
the Philox counter (coordinate group i>>3 >= 2^32), checked on sampled buckets and ranges that
the oracle computes one by one.  Inputs are generated on the device in 2^28-element chunks.
"""
import numpy as np
import pytest
import torch

from test_gpu_parity import B, S, assert_codes_equal, oracle_planes, random_packed  # noqa: F401

pytestmark = pytest.mark.gpu

CHUNK = 1 << 28


def fill_normal(t, seed, scale):
    g = torch.Generator(device="cuda").manual_seed(seed)
    flat = t.view(-1)
    for a in range(0, flat.numel(), CHUNK):
        flat[a:a + CHUNK].normal_(0.0, scale, generator=g)


def check_buckets(oracle, B, x_row, packed_row, lay, d, s, bucket, seed, rnd, worker, buckets):
    nb, _, _, N, m = oracle.shape(d, s, bucket)
    norms, sg, lv = B.planes(packed_row, lay)
    for b in buckets:
        i0, i1 = b * bucket, min((b + 1) * bucket, d)
        v = x_row[i0:i1].cpu().numpy()
        onorm, olevel, osign = oracle.quantize_bucket(v, N, i0, s, seed, rnd, worker)
        assert np.float32(onorm).tobytes() == np.float32(norms[b].item()).tobytes(), b
        sw = sg[i0 // 32:(i1 + 31) // 32].cpu().numpy().view(np.uint32)
        lw = lv[(i0 * m) // 32:(i1 * m + 31) // 32].cpu().numpy().view(np.uint32)
        osw, olw = oracle.pack(olevel, osign, s)
        assert np.array_equal(sw, osw), b
        assert np.array_equal(lw, olw), b


def need_free(gib):
    free, _ = torch.cuda.mem_get_info()
    if free < gib * (1 << 30):
        pytest.skip(f"needs {gib} GiB of free device memory")


def test_beyond_2_to_32_coordinates(oracle, B, S):
    need_free(120)
    d, K, s, bucket = (1 << 32) + 5 * 512 + 77, 2, 4, 512
    stride = (d + 63) // 64 * 64
    seed, rnd = 0x1234ABCD5678, 6
    slab = torch.empty((K, stride), dtype=torch.float32, device="cuda")
    fill_normal(slab, 17, 1e-3)
    lay = B.qesgd_layout_query(d, s, bucket)
    packed = B.alloc_packed(lay, K)
    packed.zero_()
    B.qesgd_quantize_pack_batched(slab, stride, None, d, s, bucket, 0, seed, rnd, K, packed, packed.stride(0))
    torch.cuda.synchronize()
    nb = lay.n_buckets
    edge = (1 << 32) // bucket
    rng = np.random.default_rng(5)
    buckets = sorted({0, 1, edge - 1, edge, edge + 1, nb - 2, nb - 1, *rng.integers(0, nb, size=4).tolist()})
    for k in range(K):
        check_buckets(oracle, B, slab[k], packed[k], lay, d, s, bucket, seed, rnd, k, buckets)
    del slab, packed
    torch.cuda.empty_cache()

    # server side at the same size on seeded random code planes
    lay, packed = random_packed(B, S, d, s, bucket, K, seed=9)
    w = torch.empty(d, dtype=torch.float32, device="cuda")
    fill_normal(w, 23, 0.05)
    zsum = torch.empty(d, dtype=torch.float32, device="cuda")
    fill_normal(zsum, 29, 1e-3)
    zsum0 = zsum.clone()
    zbar = torch.empty(d, dtype=torch.float32, device="cuda")
    u = torch.empty(d, dtype=torch.float32, device="cuda")
    B.qesgd_unpack_aggregate_update(packed, packed.stride(0), K, d, s, bucket, w, zbar, u, zsum)
    torch.cuda.synchronize()
    hn, hs, hl = oracle_planes(B, packed, lay, K)
    starts = [0, (1 << 32) - 3000, d - 4000, *[int(a) for a in rng.integers(0, d - 4000, size=3)]]
    for a in starts:
        e = min(d, a + 4000)
        oz = oracle.unpack_aggregate(hn, hs, hl, d, s, bucket, a, e)
        ou, ozs = oracle.apply_update(w[a:e].cpu().numpy(), oz, zsum0[a:e].cpu().numpy())
        assert np.array_equal(zbar[a:e].cpu().numpy(), oz), a
        assert np.array_equal(u[a:e].cpu().numpy(), ou), a
        assert np.array_equal(zsum[a:e].cpu().numpy(), ozs), a


def test_beyond_2_to_35_coordinates_philox_counter_high_word(oracle, B):
    need_free(160)
    d, s, bucket = (1 << 35) + 3 * 4096 + 1234, 2, 4096
    seed, rnd, worker = 0xFEDCBA9876543210, 0xFFFFFFFF, 63
    x = torch.empty(d, dtype=torch.float32, device="cuda")
    fill_normal(x, 31, 1e-2)
    lay = B.qesgd_layout_query(d, s, bucket)
    packed = B.alloc_packed(lay, 1)
    packed.zero_()
    B.qesgd_quantize_pack(x, None, d, s, bucket, 0, seed, rnd, worker, packed)
    torch.cuda.synchronize()
    nb = lay.n_buckets
    edge = (1 << 35) // bucket
    rng = np.random.default_rng(6)
    buckets = sorted({0, edge - 1, edge, edge + 2, nb - 2, nb - 1, *rng.integers(0, nb, size=4).tolist()})
    check_buckets(oracle, B, x, packed[0], lay, d, s, bucket, seed, rnd, worker, buckets)


@pytest.mark.parametrize("d,bucket,s,K,norm_kind", [
    (138_357_544, 1 << 30, 2, 2, 0),            # one bucket of 2^28 slots: 65,536 partial sums, 4 finish tiles
    ((1 << 28) + 12_345, 1 << 27, 4, 1, 0),     # buckets of 2^27: two full ones and a short one
    (70_000_003, 1 << 30, 16, 1, 1)])           # max norm over 2^27 slots (guarded passes)
def test_buckets_beyond_one_finish_tile(oracle, B, d, bucket, s, K, norm_kind):
    """Buckets with more partial sums (one per 4096 coordinates) than the 16,384 one workgroup of the
    finishing pass reduces at a time: its per-tile totals are joined like the rest of the tree.
    Every scale and code word against the oracle."""
    need_free(8)
    g = torch.Generator(device="cpu").manual_seed(d % 1000 + K)
    stride = (d + 63) // 64 * 64
    slab = torch.zeros(K, stride)
    slab[:, :d] = torch.randn(K, d, generator=g) * 1e-3
    slab[:, 12_345_678] = 0.75                      # one entry that dominates the max norm
    lay = B.qesgd_layout_query(d, s, bucket)
    wsb = B.qesgd_workspace_bytes(d, s, bucket, K)
    assert wsb // 4 // K // lay.n_buckets > 16_384
    ws = torch.full((wsb // 4,), float("nan"), device="cuda")
    packed = B.alloc_packed(lay, K)
    packed.fill_(0xA5)
    B.qesgd_quantize_pack_batched(slab.cuda(), stride, None, d, s, bucket, norm_kind, 3, 1, K, packed,
                                  packed.stride(0), ws)
    torch.cuda.synchronize()
    for k in range(K):
        assert_codes_equal(oracle, B, slab[k, :d].numpy(), s, bucket, 3, 1, k, lay, packed[k], norm_kind=norm_kind)
