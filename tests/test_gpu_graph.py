"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
caller can record them into a HIP graph.  One graph holds the dual quantizer, the group maxima and three forwards
(Alg. 1, the per-token variant with group maxima, the non-causal variant); it is replayed several times with eager work
and synchronisations between the replays, and every replay must reproduce the eager results bit for bit."""
import pytest
import torch

from paper_2604_03950_amd import workloads as wl


@pytest.mark.gpu
def test_entry_points_replay_from_a_graph():
    from paper_2604_03950_amd import binding as dma
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dma.load()
    w = wl.small_variant(wl.CONFIGS["prefill_8k"], S=1024, Hq=8, Hkv=4, B=2)
    qd, kd, vd = (dma.bits_to_bf16_tensor(a) for a in wl.generate(w))
    shape = (w.B, w.Hq, w.S, w.D)

    def enqueue(outs, quant, qam, kam):
        dma.dma_mx_quantize_dual(kd.reshape(-1, w.D), False, out=quant)
        dma.dma_mx_group_amax(qd, True, dma.GRAN_BLOCK, w.tile, out=qam)
        dma.dma_mx_group_amax(kd, False, dma.GRAN_BLOCK, w.tile, out=kam)
        dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=w.band, out=outs[0])
        dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=1, sink_tiles=1, per_token_scale=True, group_amax=(qam, kam), out=outs[1])
        dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=2, causal=False, out=outs[2])

    def buffers():
        outs = [torch.full(shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(3)]
        quant = dma.dma_mx_quantize_dual(kd.reshape(-1, w.D), False)
        quant = tuple(torch.zeros_like(t) for t in quant)
        qam = torch.zeros((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda")
        kam = torch.zeros((w.B, w.Hkv, w.S), dtype=torch.float32, device="cuda")
        return outs, quant, qam, kam

    eager = buffers()
    enqueue(*eager)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(o).all()) for o in eager[0])

    held = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(*held)                                    # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(*held)
    torch.cuda.synchronize()

    def flat(b):
        outs, quant, qam, kam = b
        return list(outs) + list(quant) + [qam, kam]

    for replay in range(4):
        for t in flat(held):
            t.fill_(0)                                    # a fill kernel, not a memset node; eager, between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(flat(held), flat(eager))):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (replay, i)
        # eager work between the replays
        again = torch.empty(shape, dtype=torch.float32, device="cuda")
        dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=w.band, out=again)
        torch.cuda.synchronize()
        assert torch.equal(again, eager[0][0])
