"""The library under HIP graph capture.  Every entry point only enqueues kernels on the caller's stream (no
allocation, no memset, no synchronisation), so a captured chain replays as a graph.  Replays are checked against
the eager results bit for bit, several times, with eager work and synchronisations of the program's own between
them; inputs are changed between replays, so a replay that did not really run the kernels would be noticed."""
import numpy as np
import pytest

import axo_synth as syn
import paper_2305_13525_amd as axo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import gpu_util as gu  # noqa: E402


def build_chain(layers, seed_shift=0):
    objs, keep = [], []
    for L in layers:
        d = syn.layer_inputs(L)
        M, Kl, Nl = L.shard
        t = {k: gu.to_dev(v) for k, v in d.items()}
        t["Y"], t["dX"], t["dW"] = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl), gu.empty_dev(Kl, Nl)
        keep.append(t)
        p = axo.Problem.make(L.grid, (0, 0, 0), L.T, L.K, L.N)
        objs.append(axo.Layer(p, L.epilogue, 0, t["X"].data_ptr(), Kl, t["W"].data_ptr(), Nl,
                              t["bias"].data_ptr() if L.epilogue else None, t["Y"].data_ptr(), Nl,
                              t["dY"].data_ptr(), Nl, t["dX"].data_ptr(), Kl, t["dW"].data_ptr(), Nl))
    return objs, keep


@pytest.mark.parametrize("entry", ["axo_layer_step", "axo_layer_step_ordered"])
def test_chain_replays_as_a_graph(entry):
    step = getattr(axo, entry)
    layers = syn.configs()["cfg5"][1:3]            # attn-out and MLP-up (+GELU) of the config-5 chain: 6 products
    objs, keep = build_chain(layers)
    db = torch.zeros(layers[1].shard[2], dtype=torch.float32, device="cuda:0")
    p1 = objs[1].p

    def enqueue(stream):
        step(objs, None, 0, stream)
        axo.axo_bias_grad_static(p1, objs[1].dY, objs[1].lddy, db.data_ptr(), 0, stream)

    def snapshot():
        torch.cuda.synchronize()
        return [t[k].clone() for t in keep for k in ("Y", "dX", "dW")] + [db.clone()]

    enqueue(gu.stream())                            # eager once: first-use set-up happens outside the capture
    want = snapshot()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enqueue(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for t in keep:                              # wipe the outputs: a replay has to write them again
            for k in ("Y", "dX", "dW"):
                t[k].fill_(0x7FC0)
        db.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device="cuda:0").sum()     # eager work of the program's own in between
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        assert all(torch.equal(a, b) for a, b in zip(got, want)), rep
        assert torch.isfinite(scratch)
    # new inputs, same graph: the replay must follow them (compare with an eager run on the new inputs)
    keep[0]["X"].copy_(gu.to_dev(syn.normal_bf16(77, 0, tuple(keep[0]["X"].shape), 1.0)))
    keep[1]["dY"].copy_(gu.to_dev(syn.normal_bf16(77, 2, tuple(keep[1]["dY"].shape), 1.0)))
    g.replay()
    got = snapshot()
    enqueue(gu.stream())
    want2 = snapshot()
    assert all(torch.equal(a, b) for a, b in zip(got, want2))
    assert not torch.equal(want2[0], want[0]) and not torch.equal(want2[-1], want[-1])
