"""A seeded sample of shapes nobody picked by hand: dimension, bucket size (power of two or not,
narrower or wider than one workgroup's tile, wider than the vector), level width, worker count,
norm, center.  Each case runs the batched quantiser, the fused aggregate/update and the one-call
round through the C ABI and compares every scale, code word and output coordinate with the oracle
(bit for bit)."""
import numpy as np
import pytest
import torch

from test_gpu_parity import B, S  # noqa: F401

pytestmark = pytest.mark.gpu

LEVELS = [2, 4, 8, 16, 32, 64, 128, 256, 65536]


def draw_case(rng):
    d = int(np.exp(rng.uniform(np.log(1), np.log(400_000))))
    kind = rng.integers(0, 4)
    if kind == 0:
        bucket = 1 << int(rng.integers(5, 18))                      # power of two, 32 .. 131072
    elif kind == 1:
        bucket = 32 * int(rng.integers(1, 3000))                    # any multiple of 32 up to 96k
    elif kind == 2:
        bucket = d + int(rng.integers(0, 1000))                     # one bucket over the whole vector
    else:
        bucket = 32 * int(rng.integers(1, 40))                      # small
    return dict(d=d, bucket=bucket, s=int(rng.choice(LEVELS)), K=int(rng.integers(1, 7)),
                norm_kind=int(rng.integers(0, 2)), center=bool(rng.integers(0, 2)), seed=int(rng.integers(1, 2**40)),
                rnd=int(rng.integers(0, 1000)))


CASES = [draw_case(np.random.default_rng(1000 + j)) for j in range(160)]


@pytest.mark.parametrize("case", CASES, ids=[f"{j}-d{c['d']}-b{c['bucket']}-s{c['s']}-K{c['K']}-n{c['norm_kind']}-c{int(c['center'])}"
                                             for j, c in enumerate(CASES)])
def test_random_shape(oracle, B, case):
    d, bucket, s, K = case["d"], case["bucket"], case["s"], case["K"]
    kind, seed, rnd = case["norm_kind"], case["seed"], case["rnd"]
    g = torch.Generator(device="cpu").manual_seed(seed % (2**31))
    stride = (d + 63) // 64 * 64
    slab = torch.zeros(K, stride)
    scale = torch.pow(10.0, torch.rand(K, 1, generator=g) * 4 - 4)
    slab[:, :d] = torch.randn(K, d, generator=g) * scale
    c = torch.randn(d, generator=g) if case["center"] else None
    if c is not None:
        slab[:, :d] += c[None, :]
    w = torch.randn(d, generator=g)
    zsum0 = torch.randn(d, generator=g) * 1e-2
    lay = B.qesgd_layout_query(d, s, bucket)
    wsb = B.qesgd_workspace_bytes(d, s, bucket, K)
    ws = torch.empty(max(wsb, 4) // 4, device="cuda") if wsb else None
    dslab = slab.cuda()
    dc = None if c is None else c.cuda()
    xs = dslab.stride(0) if K > 1 else 0

    packed = B.alloc_packed(lay, K)
    packed.fill_(0xA5)
    B.qesgd_quantize_pack_batched(dslab, xs, dc, d, s, bucket, kind, seed, rnd, K, packed, packed.stride(0), ws)
    zbar = torch.full((d,), float("nan"), device="cuda")
    u = torch.full((d,), float("nan"), device="cuda")
    zsum = zsum0.cuda()
    B.qesgd_unpack_aggregate_update(packed, packed.stride(0), K, d, s, bucket, w.cuda(), zbar, u, zsum)
    torch.cuda.synchronize()

    ch = None if c is None else c.numpy()
    planes = [oracle.quantize_pack(slab[k, :d].numpy(), s, bucket, seed, rnd, k, center=ch, norm_kind=kind)
              for k in range(K)]
    for k in range(K):
        n, sg, lv = B.planes(packed[k], lay)
        assert np.array_equal(n.cpu().numpy().view(np.uint32), planes[k][0].view(np.uint32)), (k, "scales")
        assert np.array_equal(sg.cpu().numpy().view(np.uint32), planes[k][1]), (k, "signs")
        assert np.array_equal(lv.cpu().numpy().view(np.uint32), planes[k][2]), (k, "levels")
    oz = oracle.unpack_aggregate(np.stack([p[0] for p in planes]), np.stack([p[1] for p in planes]),
                                 np.stack([p[2] for p in planes]), d, s, bucket)
    ou, ozs = oracle.apply_update(w.numpy(), oz, zsum0.numpy())
    for got, want, what in ((zbar, oz, "zbar"), (u, ou, "u"), (zsum, ozs, "zsum")):
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), what

    packed2 = B.alloc_packed(lay, K)
    packed2.fill_(0xA5)
    zbar2 = torch.full((d,), float("nan"), device="cuda")
    u2 = torch.full((d,), float("nan"), device="cuda")
    zsum2 = zsum0.cuda()
    B.qesgd_round(dslab, xs, dc, d, s, bucket, kind, seed, rnd, K, packed2, packed2.stride(0), w.cuda(), zbar2, u2,
                  zsum2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(packed2, packed)
    assert torch.equal(zbar2.view(torch.int32), zbar.view(torch.int32))
    assert torch.equal(u2.view(torch.int32), u.view(torch.int32))
    assert torch.equal(zsum2.view(torch.int32), zsum.view(torch.int32))
