"""The library allocates nothing and never synchronises, so its calls can be
captured into a HIP graph on the caller's stream.  A captured sequence of steps
must give, on every replay, exactly what the same calls give eagerly."""
import pytest
import torch

import synth
from test_gpu_parity import DEV, dirty_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    return lib


def test_steps_captured_in_a_graph_replay_bit_identically(ss):
    cfg = synth.C1                                   # the launch-bound workload is where a graph pays
    K = 5
    g = [[synth.grad_chunk(cfg, k, w, 0, DEV) for w in range(cfg.M)] for k in range(K)]
    x0 = synth.x0_chunk(cfg, 0, DEV)

    def fresh():
        return [torch.zeros(cfg.d, device=DEV) for _ in range(cfg.M)], x0.clone(), dirty_bits(ss, cfg.d)

    # eager reference: two passes over the K gradients
    m_ref, x_ref, v_ref = fresh()
    for _ in range(2):
        for k in range(K):
            ss.signum_vote_step(g[k], m_ref, cfg.beta, cfg.delta, x_ref, v_ref)
    torch.cuda.synchronize()

    m, x, voted = fresh()
    sums = torch.zeros(cfg.d, dtype=torch.int8, device=DEV)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        # warm-up outside the capture, then restore the state it touched
        ss.signum_vote_step(g[0], m, cfg.beta, cfg.delta, x, voted)
        for t in m:
            t.zero_()
        x.copy_(x0)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for k in range(K):
                ss.signum_vote_step(g[k], m, cfg.beta, cfg.delta, x, voted)
    for replay in range(2):
        graph.replay()
        torch.cuda.synchronize()
        # eager work of the program between the replays
        sums.add_(1)
        torch.cuda.synchronize()
    assert torch.equal(x.view(torch.int32), x_ref.view(torch.int32))
    assert torch.equal(voted, v_ref)
    for a, b in zip(m, m_ref):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
