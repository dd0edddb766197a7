"""The library's calls can be recorded into a HIP graph: they allocate nothing, synchronise nothing and
clear their scratch with their own kernels.  A captured step is replayed several times, with eager work and
synchronisations of the program between the replays, and every replay must reproduce the eager step bit for
bit (all kernels are deterministic)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _capture(step):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # first use outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()                                  # the binding launches on torch's current stream: the capturing one
    return graph


def _replays_match(graph, outputs, reference, before_each):
    for it in range(3):
        before_each()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in outputs().items():
            assert torch.equal(t, reference[name]), "replay %d: %s differs from the eager step" % (it, name)
        # eager work of the program between replays
        assert float(torch.arange(1000, device="cuda", dtype=torch.float32).sum()) == 499500.0


@pytest.mark.parametrize("dtype,save_logits,algorithm", [("bf16", True, 1), ("bf16", False, 1), ("f32", True, 1),
                                                         ("bf16", True, 2)])
def test_output_layer_step_in_a_graph(dtype, save_logits, algorithm):
    import paper_2411_05288_amd as vp
    N, h, V, p = 300, 256, 2304, 3
    H, Ws, labels = si.small_output_case(N, h, V, p, dtype, seed=41, labels="zipf")
    plan = vp.driver.OutputLayerPlan(to_dev(H), [to_dev(w) for w in Ws], to_dev(labels), save_logits, algorithm=algorithm)

    def outputs():
        out = {"loss": plan.loss, "loss_rows": plan.loss_rows, "dH": plan.dH}
        out.update({"dW%d" % r: w for r, w in enumerate(plan.dW)})
        return out

    plan.step()
    torch.cuda.synchronize()
    reference = {k: v.clone() for k, v in outputs().items()}

    def scribble():                              # a replay must not depend on what the buffers held
        plan.workspace.fill_(0xFF)
        plan.dH.fill_(float("nan"))
        for w in plan.dW:
            w.fill_(float("nan"))

    _replays_match(_capture(plan.step), outputs, reference, scribble)


def test_embedding_step_in_a_graph():
    import paper_2411_05288_amd as vp
    N, h, V, p = 3000, 96, 512, 2
    Vs = V // p
    tables = [si.normal((Vs, h), 0.02, "bf16", 43, si.STREAM_TABLE, r) for r in range(p)]
    gout = si.normal((N, h), 1.0, "bf16", 43, si.STREAM_GRAD)
    ids = si.zipf_ids(N, V, 1.1, 43)
    plan = vp.driver.EmbeddingPlan([to_dev(t) for t in tables], to_dev(ids), to_dev(gout))

    def step():
        plan.forward()
        plan.backward()

    def outputs():
        out = {"out%d" % r: t for r, t in enumerate(plan.out)}
        out.update({"dtable%d" % r: t for r, t in enumerate(plan.dtable)})
        return out

    def reset():                                 # the scatter-add accumulates: start every step from zero
        plan.workspace.fill_(0xFF)
        for t in plan.dtable:
            t.zero_()

    reset()
    step()
    torch.cuda.synchronize()
    reference = {k: v.clone() for k, v in outputs().items()}
    assert any(float(t.abs().max()) > 0 for t in plan.dtable)
    _replays_match(_capture(lambda: (reset(), step())), outputs, reference, lambda: None)
