"""The C-ABI calls neither allocate nor synchronise and clear nothing with memset calls, so a whole
forward + backward step of the block loop can be captured in a HIP graph and replayed.  Every
replay is checked against the eager result, with eager work and synchronisations between the
replays."""
import pytest
import torch

from paper_2502_02406_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("masked", [False, True])
def test_step_replays_from_a_graph(masked):
    from paper_2502_02406_amd.blockloop import BlockLoop, MediaMask
    kw = dict(q_chunk=32, kv_block=256) if masked else {}
    w = W.Workload("graph", B=1, Hq=8, Hkv=2, D=128, Sq=200, Skv=2048, dtype="bf16", std=0.5,
                   n_blocks=1 if masked else 2, **kw)
    x = W.make_inputs(w)
    dev = {n: t.cuda() for n, t in x.items()}
    mask = MediaMask(dev["allow"], w.q_chunk, w.kv_block) if masked else None
    loop = BlockLoop(tuple(dev["q"].shape), tuple(dev["k"].shape), torch.bfloat16, w.n_blocks, mask)
    q, k, v, g = dev["q"], dev["k"], dev["v"], dev["do"]
    dk, dv = torch.empty_like(k), torch.empty_like(v)

    def step():
        o, lse = loop.forward(q, k, v)
        return o, lse, loop.backward(q, k, v, o, lse, g, dk, dv)

    o, lse, dq = step()                      # eager: also the first-call set-up of every kernel
    torch.cuda.synchronize()
    want = [t.clone() for t in (o, lse, dq, dk, dv)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                               # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for r in range(3):
        for t in (loop.o, loop.lse, loop.dq, dk, dv):      # eager work between the replays
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("O", "L", "dQ", "dK", "dV"), (loop.o, loop.lse, loop.dq, dk, dv), want):
            assert torch.equal(got, ref), f"replay {r}: {name} differs from the eager result"
