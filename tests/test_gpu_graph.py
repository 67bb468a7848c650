"""The library enqueues kernels only - no allocation, no memset, no host
synchronisation - so a call can be recorded into a HIP graph and replayed.
Each replay is checked bit for bit against the eager result, with eager work of
the library and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2511_18868_amd import synth

pytestmark = pytest.mark.gpu

OUT = ("bound", "alive", "assign", "cent", "counts", "objective", "Ncs", "mu", "ucb", "sel")


@pytest.fixture(scope="module")
def kb():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_18868_amd import binding
    binding.lib()
    return binding


CASES = {
    # one-workgroup kernels, 768-thread shape (a single launch sequence without the ordering kernel)
    "cfg2": lambda: synth.config2(iters=6),
    # one-workgroup kernels, 256-thread shape
    "manysmall": lambda: synth.config5(G=300, nmin=64, nmax=260, D=16, S=4, iters=6, seed=123),
    # the multi-workgroup launch sequence (four launches per Lloyd step)
    "cfg4s": lambda: synth.config4(N=8192, K=256, ncentres=256, iters=4),
    # very short searches: the whole round is one launch, a wave per search
    "paperscale": lambda: synth.paper_scale(),
}


@pytest.mark.parametrize("name", list(CASES))
def test_round_replays_from_a_graph(kb, name):
    import torch
    b = CASES[name]()
    d = kb.DeviceBatch(b)
    d.round()
    torch.cuda.synchronize()
    want = {k: d.host(k).copy() for k in OUT}

    def clear():
        for k in OUT:
            getattr(d, k).zero_()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    clear()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        d.round()                      # recorded on the capturing stream, not run
    torch.cuda.synchronize()
    for rep in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in OUT:
            np.testing.assert_array_equal(d.host(k).view(np.uint8), want[k].view(np.uint8),
                                          err_msg=f"{name} replay {rep}: {k}")
        # eager work of the library on the same buffers between the replays
        d.cluster()
        d.ucb_select()
        torch.cuda.synchronize()
