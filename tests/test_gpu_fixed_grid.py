"""Parity of the paper-literal fixed-grid quantiser, its fused inverse, the epoch commit and the
server-to-worker direction (HIP through the C ABI) against the CPU oracle."""
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


def gpu_quantize_fixed(B, x, delta, b, seed, rnd, worker, center=None):
    d = x.numel()
    words = (d * b + 31) // 32
    codes = torch.full((words + 8,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    B.qesgd_quantize_fixed(x, center, d, delta, b, seed, rnd, worker, codes)
    torch.cuda.synchronize()
    host = codes.cpu().numpy().view(np.uint32)
    assert (host[words:] == 0x5A5A5A5A).all()          # nothing written past the last word
    return codes, host[:words].copy()


@pytest.mark.parametrize("b", [2, 4, 8, 16])
@pytest.mark.parametrize("d", [1, 7, 8, 9, 31, 33, 511, 512, 513, 4095, 4096, 4097, 4099, 8192, 100_003, 1_000_000])
def test_quantize_fixed_matches_oracle(oracle, B, b, d):
    g = torch.Generator(device="cpu").manual_seed(d + b)
    x = (torch.randn(d, generator=g) * 1e-3).to(torch.float32)
    x[::17] *= 40.0                                     # some values beyond the range: clamp cases
    if d > 20:
        x[5] = 0.0
        x[6] = -0.0
        x[7] = 1e-12
        x[9] = -1e-12                                   # tiny negative: frac rounds to 1
    delta = float(np.float32(2e-3 / (2 ** (b - 1))))
    _, got = gpu_quantize_fixed(B, x.cuda(), delta, b, 0xABCDEF12345, 3, 11)
    want = oracle.quantize_fixed(x.numpy(), delta, b, 0xABCDEF12345, 3, 11)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"code words differ at {bad[:5]}"


def _steps_for_division():
    one = np.float32(1.0)
    out = [np.float32(2.0 ** -12), np.nextafter(np.float32(2.0 ** -10), np.float32(0)),      # significand all ones
           np.nextafter(np.float32(2.0 ** -10), one), np.float32(3.0e-4), np.float32(1.0 / 3.0), np.float32(7.77e-7),
           np.float32(2.0 ** -60), np.nextafter(np.float32(2.0 ** -60), np.float32(0)),      # both sides of the switch
           np.float32(2.0 ** 60), np.nextafter(np.float32(2.0 ** 60), np.float32(np.inf)),
           np.float32(1e-30), np.float32(1e30), np.float32(1e-38), np.float32(1e-41), np.float32(3e38)]
    return [float(x) for x in out]


@pytest.mark.parametrize("b", [2, 8, 16])
@pytest.mark.parametrize("delta", _steps_for_division())
def test_quantize_fixed_division_is_ieee_for_every_step(oracle, B, b, delta):
    """The kernel divides by the step with a reciprocal computed once where that is exact and with
    the full IEEE division elsewhere; the codes must equal the oracle's (which divides coordinate
    by coordinate) for steps on both sides of the switch, steps whose significand is all ones, and
    values from subnormal to far beyond the range."""
    d = 1 << 19
    g = torch.Generator(device="cpu").manual_seed(int(b * 1000 + abs(hash(delta)) % 997))
    half = float(2 ** (b - 1))
    u = torch.rand(d, generator=g, dtype=torch.float64) * 2 - 1
    scale = torch.empty(d, dtype=torch.float64)
    scale[0::4] = 1.0                                   # inside the range
    scale[1::4] = 2.0 ** -20                            # near zero: floor 0 or -1
    scale[2::4] = torch.pow(2.0, -(torch.rand(d // 4, generator=g, dtype=torch.float64) * 140))   # down to the subnormals of the quotient
    scale[3::4] = torch.pow(2.0, torch.rand(d // 4, generator=g, dtype=torch.float64) * 100)      # far beyond the range
    x64 = u * scale * half * delta
    x = x64.clamp(-3.0e38, 3.0e38).to(torch.float32)
    x[7] = 0.0
    x[15] = -0.0
    x[23] = 1e-45
    x[31] = -1e-45
    _, got = gpu_quantize_fixed(B, x.cuda(), delta, b, 31337, 1, 2)
    want = oracle.quantize_fixed(x.numpy(), delta, b, 31337, 1, 2)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"delta={delta!r}: code words differ at {bad[:5]}"


@pytest.mark.parametrize("b", [2, 4, 8, 16])
def test_quantize_fixed_with_center_and_grid_values(oracle, B, b):
    d = 50_001
    g = torch.Generator(device="cpu").manual_seed(b)
    w = torch.randn(d, generator=g)
    delta = 2.0 ** -12
    k = torch.randint(-(2 ** (b - 1)), 2 ** (b - 1), (d,), generator=g)
    x = w + (k.to(torch.float32) * delta)               # deviations near the grid (w + k*delta rounds)
    _, got = gpu_quantize_fixed(B, x.cuda(), delta, b, 5, 0, 1, center=w.cuda())
    want = oracle.quantize_fixed(x.numpy(), delta, b, 5, 0, 1, center=w.numpy())
    assert np.array_equal(got, want)
    # exactly on the grid without a center: the codes are k itself, whatever the variates
    xg = (k.to(torch.float32) * delta)
    _, got = gpu_quantize_fixed(B, xg.cuda(), delta, b, 6, 0, 1)
    z, _, _ = oracle.dequantize_fixed_update(got, d, delta, b)
    assert np.array_equal(z, xg.numpy())


@pytest.mark.parametrize("b", [2, 4, 8, 16])
@pytest.mark.parametrize("d", [1, 3, 4, 5, 1023, 1024, 1025, 77_777])
def test_dequantize_fixed_update_matches_oracle(oracle, B, b, d):
    from paper_1901_03040_amd import synth
    words = (d * b + 31) // 32
    codes = synth.random_packed_words(words, 99 + b, d % 1000, "cuda")
    g = torch.Generator(device="cpu").manual_seed(d)
    w = torch.randn(d, generator=g)
    zs0 = torch.randn(d, generator=g) * 1e-2
    delta = 3.1e-4
    z = torch.full((d,), float("nan"), device="cuda")
    u = torch.full((d,), float("nan"), device="cuda")
    zs = zs0.cuda()
    B.qesgd_dequantize_fixed_update(codes, d, delta, b, w.cuda(), z, u, zs)
    torch.cuda.synchronize()
    oz, ou, ozs = oracle.dequantize_fixed_update(codes.cpu().numpy().view(np.uint32), d, delta, b,
                                                 w_snap=w.numpy(), zsum=zs0.numpy())
    for got, want, what in [(z, oz, "z"), (u, ou, "u"), (zs, ozs, "zsum")]:
        got = got.cpu().numpy()
        assert float(np.max(np.abs(got - want))) <= 1e-6 * float(np.max(np.abs(want))), what
        assert np.array_equal(got, want), what
    # optional outputs
    u2 = torch.empty(d, device="cuda")
    B.qesgd_dequantize_fixed_update(codes, d, delta, b, w.cuda(), None, u2, None)
    z2 = torch.empty(d, device="cuda")
    B.qesgd_dequantize_fixed_update(codes, d, delta, b, None, z2, None, None)
    torch.cuda.synchronize()
    assert torch.equal(u2, u) and torch.equal(z2, z)


@pytest.mark.parametrize("rounds", [1, 3, 8, 10])
@pytest.mark.parametrize("d", [1, 5, 1024, 100_003])
def test_epoch_commit_matches_oracle(oracle, B, rounds, d):
    g = torch.Generator(device="cpu").manual_seed(d + rounds)
    w = torch.randn(d, generator=g)
    zsum = torch.randn(d, generator=g) * 1e-2
    wd, zd = w.cuda(), zsum.cuda()
    B.qesgd_epoch_commit(wd, zd, rounds, d)
    torch.cuda.synchronize()
    ow, oz = oracle.epoch_commit(w.numpy(), zsum.numpy(), rounds)
    assert np.array_equal(wd.cpu().numpy(), ow) and not zd.any()


def test_server_to_worker_direction(oracle, B):
    """Alg. 3, server task: the aggregated z is quantised once and sent; workers form u = w_t + Q(z).
    The same kernels with one "worker": quantize_pack of z, unpack with K = 1."""
    from paper_1901_03040_amd import synth
    cfg = synth.by_name("cfg2").scaled(d=70_001, K=1)
    z = synth.worker_vector(cfg, 0, "cuda")
    w = synth.snapshot(cfg, "cuda")
    lay = B.qesgd_layout_query(cfg.d, cfg.s, cfg.bucket)
    packed = B.alloc_packed(lay, 1)
    server_id = 63
    B.qesgd_quantize_pack(z, None, cfg.d, cfg.s, cfg.bucket, 0, 7, 2, server_id, packed)
    u = torch.empty(cfg.d, device="cuda")
    qz = torch.empty(cfg.d, device="cuda")
    B.qesgd_unpack_aggregate_update(packed, packed.stride(0), 1, cfg.d, cfg.s, cfg.bucket, w, qz, u, None)
    torch.cuda.synchronize()
    on, osw, olw = oracle.quantize_pack(z.cpu().numpy(), cfg.s, cfg.bucket, 7, 2, server_id)
    oq = oracle.unpack_aggregate(on[None], osw[None], olw[None], cfg.d, cfg.s, cfg.bucket)
    ou, _ = oracle.apply_update(w.cpu().numpy(), oq, None)
    assert np.array_equal(qz.cpu().numpy(), oq) and np.array_equal(u.cpu().numpy(), ou)


def test_fixed_grid_full_size_sampled(oracle, B):
    """cfg4's shape (d = 25,557,032, b = 8: the paper's 8-bit setting): sampled words against the oracle."""
    from paper_1901_03040_amd import synth
    cfg = synth.by_name("cfg4")
    x = synth.worker_vector(cfg, 0, "cuda")
    d, b, delta = cfg.d, 8, float(np.float32(4e-3 / 128))
    codes, host = gpu_quantize_fixed(B, x, delta, b, 21, 1, 0)
    rng = np.random.default_rng(0)
    for a in sorted({0, d - 4096, *[int(v) // 8 * 8 for v in rng.integers(0, d - 4096, size=6)]}):
        e = min(d, a + 4096)
        seg = x[a:e].cpu().numpy()
        want = np.zeros((e - a + 3) // 4, np.uint32)
        for j, v in enumerate(seg):
            k = oracle.fixed_round(v, delta, b, oracle.uniform16(21, 1, 0, a + j))
            want[j // 4] |= np.uint32((k & 0xFF) << (8 * (j % 4)))
        assert np.array_equal(host[a // 4:a // 4 + want.size], want), a
    w = synth.snapshot(cfg, "cuda")
    z = torch.empty(d, device="cuda")
    u = torch.empty(d, device="cuda")
    zsum = torch.zeros(d, device="cuda")
    B.qesgd_dequantize_fixed_update(codes, d, delta, b, w, z, u, zsum)
    torch.cuda.synchronize()
    assert torch.equal(zsum, z)
    inside = x.abs() < delta * 127
    assert float((z - x)[inside].abs().max()) <= delta * (1 + 1e-5)     # round trip stays within one step
    # the inverse at the same size on seeded random code words, sampled ranges against the oracle
    rcodes = synth.random_packed_words((d * b + 31) // 32, 5, 0, "cuda")
    B.qesgd_dequantize_fixed_update(rcodes, d, delta, b, w, z, u, None)
    torch.cuda.synchronize()
    rhost = rcodes.cpu().numpy().view(np.uint32)
    for a in (0, d - 5000, 12_345_676):
        oz, ou, _ = oracle.dequantize_fixed_update(rhost[a // 4:(a + 5000) // 4], 5000, delta, b,
                                                   w_snap=w[a:a + 5000].cpu().numpy())
        assert np.array_equal(z[a:a + 5000].cpu().numpy(), oz) and np.array_equal(u[a:a + 5000].cpu().numpy(), ou)
