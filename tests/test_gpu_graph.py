"""The library under HIP graph capture: every entry point only launches kernels on the stream it is given
(no allocation, no synchronisation, no memset or copy), so a captured sequence must replay to the bits of
the eager calls, on every replay, with eager work and synchronisations of the program in between."""
import pytest
import torch

from paper_2204_07143_amd import binding as na
from paper_2204_07143_amd import synth

from gpu_util import Stages

pytestmark = pytest.mark.gpu


def _run_everything(st: Stages):
    st.forward_unfused()
    st.forward_fused()
    st.backward_unfused()
    c = st.backward_composed()
    f = st.backward_fused()
    return [st.logits, st.attn, st.out, st.out_fused, st.lse, st.dp, st.dv, st.ds, st.dq, st.dk, st.d_rpb, *c[:4], *f]


@pytest.mark.parametrize("k,dtype", [(7, "f16"), (5, "bf16"), (9, "f16"), (3, "f32")])
def test_graph_replays_match_eager(k, dtype):
    p = synth.Problem(5, 2, 27, 41, 32, k, dtype)
    host = synth.make_inputs(p, seed=60 + k)
    st = Stages(p, host)
    eager = [t.clone() for t in _run_everything(st)]   # also the warm-up: code objects loaded, LDS limits set
    torch.cuda.synchronize()

    # the captured calls write into buffers that live as long as the graph
    class Holder(Stages):
        pass
    gst = Holder(p, host)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        outs = _run_everything(gst)
    for replay in range(4):
        for t in outs:
            t.fill_(float("nan")) if t.is_floating_point() else t.zero_()
        # eager work of the program between the replays, on the same stream, and a synchronisation
        other = _run_everything(st)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(outs, eager)):
            assert torch.equal(a, b), f"replay {replay}: output {i} differs from the eager result"
        for i, (a, b) in enumerate(zip(other, eager)):
            assert torch.equal(a, b), f"replay {replay}: eager output {i} changed"


def test_noalloc_entry_point_under_capture():
    p = synth.Problem(4, 2, 20, 33, 32, 7, "f16")
    host = synth.make_inputs(p, seed=8)
    st = Stages(p, host)
    st.forward_unfused(); st.backward_unfused()
    nb = 2 * p.k - 1
    out = torch.empty((p.heads, nb, nb), dtype=torch.float32, device="cuda")
    na.na2d_qk_bwd_rpb_noalloc(st.ds, p.k, st.q, out)   # first use on the device: looks up the array's address
    torch.cuda.synchronize()
    assert torch.equal(out, st.d_rpb)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        na.na2d_qk_bwd_rpb_noalloc(st.ds, p.k, st.q, out)
    for _ in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, st.d_rpb)
