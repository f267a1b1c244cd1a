"""The entry point that allocates nothing (qesgd_quantize_pack_batched_noalloc): through the C ABI,
its packed output equals qesgd_quantize_pack_batched's bit for bit, on calls made back to back on
the same GPU -- the second with a smaller input, so that the shared static scratch still holds the
first call's partial sums -- for dense and non-dense wide buckets, both norms, and a shape that
needs no scratch at all."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1901_03040_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()
    return binding


def both_ways(B, d, s, bucket, K, norm_kind, seed, rnd, with_center):
    g = torch.Generator(device="cpu").manual_seed(d + 7 * K + s)
    stride = (d + 63) // 64 * 64
    slab = torch.zeros(K, stride)
    slab[:, :d] = torch.randn(K, d, generator=g) * 1e-3
    slab = slab.cuda()
    center = (torch.randn(d, generator=g) * 1e-3).cuda() if with_center else None
    lay = B.qesgd_layout_query(d, s, bucket)
    ref = B.alloc_packed(lay, K)
    got = B.alloc_packed(lay, K)
    ref.fill_(0xA5)
    got.fill_(0xA5)
    wsb = B.qesgd_workspace_bytes(d, s, bucket, K)
    ws = torch.empty(max(wsb, 4) // 4, dtype=torch.float32, device="cuda") if wsb else None
    B.qesgd_quantize_pack_batched(slab, stride, center, d, s, bucket, norm_kind, seed, rnd, K, ref, ref.stride(0), ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.qesgd_quantize_pack_batched_noalloc(slab, stride, center, d, s, bucket, norm_kind, seed, rnd, K, got,
                                          got.stride(0))
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert wsb <= B.NOALLOC_SCRATCH_BYTES
    return wsb, torch.equal(ref, got), ref


def test_noalloc_equals_workspace_form_on_consecutive_calls(B):
    # first a large call (1024 partial sums per worker), then smaller ones that reuse the scratch
    calls = [
        (2_100_001, 16, 1 << 30, 3, 0, False),     # one bucket over the whole vector, ragged last tile
        (300_001, 4, 262_144, 3, 0, True),         # two wide power-of-two buckets, with center
        (200_003, 256, 48_000, 2, 0, False),       # wide bucket that is not a power of two
        (100_000, 2, 100_000, 2, 1, False),        # max norm
        (150_000, 32, 65_536, 3, 0, False),        # level width that does not divide a word
        (50_000, 16, 512, 4, 0, False),            # needs no scratch
        (100_000, 2, 100_000, 1, 0, True),         # one worker
    ]
    needs = []
    for n, (d, s, bucket, K, kind, cen) in enumerate(calls):
        print(f"noalloc case {n}: d={d} s={s} bucket={bucket} K={K} kind={kind} center={cen}", flush=True)
        wsb, same, _ = both_ways(B, d, s, bucket, K, kind, 77, n, cen)
        needs.append(wsb)
        assert same, (d, s, bucket, K, kind, cen)
    assert needs[0] > needs[1] > 0 and needs[5] == 0


def test_noalloc_matches_oracle(oracle, B):
    """The same two calls checked against the oracle directly, second smaller than the first."""
    import numpy as np
    for rnd, (d, s, bucket, K) in enumerate([(700_001, 16, 1 << 30, 2), (90_001, 16, 1 << 30, 2)]):
        g = torch.Generator(device="cpu").manual_seed(d)
        stride = (d + 63) // 64 * 64
        slab = torch.zeros(K, stride)
        slab[:, :d] = torch.randn(K, d, generator=g) * 1e-3
        lay = B.qesgd_layout_query(d, s, bucket)
        got = B.alloc_packed(lay, K)
        B.qesgd_quantize_pack_batched_noalloc(slab.cuda(), stride, None, d, s, bucket, 0, 5, rnd, K, got, got.stride(0))
        torch.cuda.synchronize()
        for k in range(K):
            n, sg, lv = B.planes(got[k], lay)
            on, osw, olw = oracle.quantize_pack(slab[k, :d].numpy(), s, bucket, 5, rnd, k)
            assert np.array_equal(n.cpu().numpy().view(np.uint32), on.view(np.uint32))
            assert np.array_equal(sg.cpu().numpy().view(np.uint32), osw)
            assert np.array_equal(lv.cpu().numpy().view(np.uint32), olw)


def test_noalloc_rejects_shapes_beyond_the_scratch(B):
    d, K = 1 << 31, 4                                   # 4 x 2^31 / 4096 partial sums = 8 MiB
    assert B.qesgd_workspace_bytes(d, 2, d, K) > B.NOALLOC_SCRATCH_BYTES
    rc = B.lib().qesgd_quantize_pack_batched_noalloc(0x10000, d, None, d, 2, d, 0, 1, 0, K, 0x20000, 1 << 33, None)
    assert rc == B.ERR_SCRATCH
    assert "scratch" in B.strerror(rc)
