"""The library under HIP graph capture (no allocation, no synchronisation, no memset inside a
call) and checkpoint / resume of a multi-round run (the variates are stateless: resuming is
passing the same (seed, round))."""
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


@pytest.fixture(scope="module")
def S():
    from paper_1901_03040_amd import synth
    return synth


@pytest.mark.parametrize("form", ["two_calls", "one_call", "noalloc_wide_bucket", "two_calls_wide_bucket"])
def test_round_replays_from_a_graph(B, S, form):
    """One round captured in a graph and replayed with eager work in between, in the two-call form,
    through qesgd_round (one launch), and with a whole-vector scale (several launches per call)
    through the entry point that takes no workspace and the one that does."""
    wide = form.endswith("wide_bucket")
    cfg = S.by_name("cfg2").scaled(d=300_003, K=4, bucket=(1 << 30) if wide else None)
    slab = S.worker_slab(cfg, "cuda")
    wsb = B.qesgd_workspace_bytes(cfg.d, cfg.s, cfg.bucket, cfg.K)
    assert (wsb > 0) == wide
    ws = torch.empty(max(wsb, 4) // 4, device="cuda")
    w = S.snapshot(cfg, "cuda")
    lay = B.qesgd_layout_query(cfg.d, cfg.s, cfg.bucket)

    def buffers():
        return (B.alloc_packed(lay, cfg.K).zero_(), torch.zeros(cfg.d, device="cuda"),
                torch.zeros(cfg.d, device="cuda"), torch.zeros(cfg.d, device="cuda"))

    def reference_round(packed, zbar, u, zsum, rnd):
        B.qesgd_quantize_pack_batched(slab, slab.stride(0), None, cfg.d, cfg.s, cfg.bucket, 0, cfg.seed, rnd,
                                      cfg.K, packed, packed.stride(0), ws if wide else None)
        B.qesgd_unpack_aggregate_update(packed, packed.stride(0), cfg.K, cfg.d, cfg.s, cfg.bucket, w, zbar, u, zsum)

    def one_round(packed, zbar, u, zsum, rnd):
        if form == "one_call":
            B.qesgd_round(slab, slab.stride(0), None, cfg.d, cfg.s, cfg.bucket, 0, cfg.seed, rnd, cfg.K, packed,
                          packed.stride(0), w, zbar, u, zsum)
            return
        if form == "noalloc_wide_bucket":
            B.qesgd_quantize_pack_batched_noalloc(slab, slab.stride(0), None, cfg.d, cfg.s, cfg.bucket, 0, cfg.seed,
                                                  rnd, cfg.K, packed, packed.stride(0))
            B.qesgd_unpack_aggregate_update(packed, packed.stride(0), cfg.K, cfg.d, cfg.s, cfg.bucket, w, zbar, u, zsum)
            return
        reference_round(packed, zbar, u, zsum, rnd)

    # eager reference: the same round three times (zsum accumulates 1x, 2x, 3x)
    ep, ez, eu, es = buffers()
    eager = []
    for _ in range(3):
        reference_round(ep, ez, eu, es, 7)
        torch.cuda.synchronize()
        eager.append((ep.clone(), ez.clone(), eu.clone(), es.clone()))

    gp, gz, gu, gs = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_round(gp, gz, gu, gs, 7)                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gs.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_round(gp, gz, gu, gs, 7)
    for i in range(3):
        graph.replay()
        torch.cuda.synchronize()
        # eager work of the program between replays
        scratch = torch.randn(1 << 20, device="cuda").sum().item()
        assert np.isfinite(scratch)
        for got, want in zip((gp, gz, gu, gs), eager[i]):
            assert torch.equal(got, want), i


def test_resume_in_the_middle_gives_identical_bytes(B, S):
    cfg = S.by_name("cfg3").scaled(d=123_457, K=4)
    slab = S.worker_slab(cfg, "cuda")
    w0 = S.snapshot(cfg, "cuda")
    lay = B.qesgd_layout_query(cfg.d, cfg.s, cfg.bucket)

    def run(first, last, state):
        w, zsum = state
        packed = B.alloc_packed(lay, cfg.K).zero_()       # the gaps between the planes are never written
        zbar = torch.empty(cfg.d, device="cuda")
        u = torch.empty(cfg.d, device="cuda")
        rot = torch.empty_like(slab)
        for rnd in range(first, last):
            rot.copy_(slab[[(k + rnd) % cfg.K for k in range(cfg.K)]])
            B.qesgd_quantize_pack_batched(rot, rot.stride(0), None, cfg.d, cfg.s, cfg.bucket, 0, cfg.seed, rnd,
                                          cfg.K, packed, packed.stride(0))
            B.qesgd_unpack_aggregate_update(packed, packed.stride(0), cfg.K, cfg.d, cfg.s, cfg.bucket, w, zbar, u, zsum)
        B.qesgd_epoch_commit(w, zsum, last - first, cfg.d) if last == 10 and first == 0 else None
        torch.cuda.synchronize()
        return packed, u, zsum, w

    straight = run(0, 10, (w0.clone(), torch.zeros(cfg.d, device="cuda")))
    # first half, "checkpoint" to the host, second half from the restored state
    _, _, zsum5, w5 = run(0, 5, (w0.clone(), torch.zeros(cfg.d, device="cuda")))
    ckpt = (w5.cpu(), zsum5.cpu())
    packed, u, zsum, w = run(5, 10, (ckpt[0].cuda(), ckpt[1].cuda()))
    B.qesgd_epoch_commit(w, zsum, 10, cfg.d)
    torch.cuda.synchronize()
    for got, want in zip((packed, u, zsum, w), straight):
        assert torch.equal(got, want)
