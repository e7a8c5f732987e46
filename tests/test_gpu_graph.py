"""A whole n-wise step captured into a HIP graph (both of the library's streams, their event
fork / joins) and replayed: every replay must give the eager step's results bit for bit.  The
library creates its second stream and all events during the first eager step, records no
memset, and allocates nothing, so the five calls can be captured as they are."""
import numpy as np
import pytest

from paper_2010_04116_amd import binding, synth
from parity import make_inputs

pytestmark = pytest.mark.gpu


def _all_equal(w, a, b, what):
    assert np.array_equal(a["losses"], b["losses"]), what
    assert np.array_equal(a["dx0"], b["dx0"]), what
    for k in range(w.K):
        assert np.array_equal(a["head_grads"][k], b["head_grads"][k]), (what, k)
        for l in range(w.L):
            for name in synth.BLOCK_TENSORS:
                assert np.array_equal(a["comp_grads"][k][l][name], b["comp_grads"][k][l][name]), (what, k, l, name)


@pytest.mark.parametrize("name,static_heads", [("bits", False), ("small", False), ("bits", True)])
def test_graph_replays_equal_the_eager_step(name, static_heads):
    """static_heads: the heads run through il_head_xent_static (scratch in the library's static device
    array, everything in line on the captured stream) - the entry point meant for callers under capture."""
    import torch
    if name == "small":
        w = synth.WORKLOADS["small"]
    else:
        w = synth.Workload("bits", "bf16", K=3, L=3, d=256, H=4, m=1024, V=2048, B=2, T=128, n=2)
    params, x0, tgt = make_inputs(w, seed=31)
    _, x0b, tgtb = make_inputs(w, seed=32)
    stream = torch.cuda.Stream()
    st = binding.Step(w, binding.pack_params(w, params), stream=stream)
    with torch.cuda.stream(stream):
        st.set_inputs(x0, tgt)
        st.run(static_heads)                       # eager: also creates the library's stream and events
        eager = st.results()
        st.set_inputs(x0b, tgtb)
        st.run(static_heads)
        eager_b = st.results()
    stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        st.run(static_heads)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        for rep in range(3):
            inputs, want = ((x0, tgt), eager) if rep != 1 else ((x0b, tgtb), eager_b)
            st.set_inputs(*inputs)                 # eager work between the replays
            st.grads.fill_(7.0)                    # every gradient element is rewritten by the replay
            st.losses.zero_()
            g.replay()
            _all_equal(w, st.results(), want, f"{name} replay {rep}")
            st.run(static_heads)                   # and an eager step on the same context afterwards
            _all_equal(w, st.results(), want, f"{name} eager after replay {rep}")
    del g
    st.close()
