"""The compute calls only enqueue kernels (no allocation, no host synchronisation, no memset), so a
caller may capture them into a HIP graph; a selector call that would have to probe is refused during capture.  The graph is replayed several times with fresh inputs
and eager work in between, and every replay is compared bit for bit with the eager result."""
import numpy as np
import pytest

from paper_2511_17594_amd import workloads as W
from util import dev

pytestmark = pytest.mark.gpu


def test_spmm_sddmm_attention_replay_from_a_captured_graph():
    import torch
    from paper_2511_17594_amd import binding as ab

    A = W.config2_powerlaw(n=20000, mean_deg=20.0, dmax=4096, seed=9)
    N, nnz, F, H, d = A.n_rows, A.nnz, 64, 4, 32
    h = ab.Handle(0)
    rp, ci, va = dev(A.rowptr, torch), dev(A.colind, torch), dev(A.val, torch)
    B = torch.randn(N, F, device="cuda")
    X = torch.randn(N, F, device="cuda")
    Q, K, V = (torch.randn(N, H, d, device="cuda").to(torch.bfloat16) for _ in range(3))
    C = torch.empty(N, F, device="cuda")
    out = torch.empty(nnz, device="cuda")
    O = torch.empty(N, H, d, device="cuda")
    s_hub = ab.Schedule(mapping=ab.MAP_WAVE_ROW, hub_t=256, hub_chunk=256)
    s_att = ab.Schedule(mapping=ab.MAP_FUSED, hub_t=256, hub_chunk=256)
    ws1 = torch.empty(h.workspace_bytes(ab.OP_SPMM, N, nnz, F, 1, s_hub), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(h.workspace_bytes(ab.OP_SPMM, N, nnz, F), dtype=torch.uint8, device="cuda")
    ws3 = torch.empty(h.workspace_bytes(ab.OP_ATTENTION, N, nnz, d, H, s_att), dtype=torch.uint8, device="cuda")

    def work(stream):
        h.spmm(N, N, rp, ci, va, B, C, F, sched=s_hub, workspace=ws1, stream=stream)        # explicit schedule
        h.sddmm(N, N, rp, ci, X, B, out, F, workspace=ws2, stream=stream)                   # selector, replayed from cache
        h.csr_attention(N, rp, ci, Q, K, V, O, H, d, d ** -0.5, sched=s_att, workspace=ws3, stream=stream)

    work(torch.cuda.current_stream())          # warm: the selector probes and caches outside the capture
    torch.cuda.synchronize()
    assert h.last_decision() is not None
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        work(side)                             # once more on the capture stream before capturing
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            work(torch.cuda.current_stream())
            # a decision that would need probes (SpMM at this width was never decided) is refused while the stream
            # is being captured, before anything touches the stream: the capture stays valid
            with pytest.raises(ab.AutosageError) as refused:
                h.spmm(N, N, rp, ci, va, B, C, F, workspace=ws2, stream=torch.cuda.current_stream())
            assert refused.value.status == ab.ERR_UNSUPPORTED
    torch.cuda.synchronize()

    for rep in range(3):
        gen = torch.Generator(device="cuda").manual_seed(100 + rep)
        B.copy_(torch.randn(N, F, device="cuda", generator=gen))
        X.copy_(torch.randn(N, F, device="cuda", generator=gen))
        K.copy_(torch.randn(N, H, d, device="cuda", generator=gen).to(torch.bfloat16))
        work(torch.cuda.current_stream())      # eager reference (bit-reproducible for a fixed schedule)
        torch.cuda.synchronize()
        ref = [t.clone() for t in (C, out, O)]
        for t in (C, out, O):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, ref[0]) and torch.equal(out, ref[1]) and torch.equal(O, ref[2]), rep
    h.close()
