"""GPU parity at the benchmark's full shard sizes, in the launch configuration bench.py times
(contiguous shards, coordinate (0,0,0), axo_layer_step for the chain: one dependence level, grouped launches).  The fp64 oracle computes
a stratified sample of whole output rows (first and last row of every 256-row block plus one seeded
row out of every 16, so every 16-row band of every matrix-core tile of every workgroup tile is hit and,
since rows are whole, every tile column).  Configs 2, 3, 4 and 5 through axo_layer_step are compared on ALL rows,
every element (the oracle needs 5-14 s per config on the GPU host's 16 cores); the ordered chain and the GPT-20B
block, whose oracle would take minutes, on the sample."""
import numpy as np
import pytest

import axo_synth as syn
import oracle
import paper_2305_13525_amd as axo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import gpu_util as gu  # noqa: E402


def run_chain(layers, step=None):
    step = step or axo.axo_layer_step
    objs, keep = [], []
    for L in layers:
        d = syn.layer_inputs(L)
        M, Kl, Nl = L.shard
        t = {k: gu.to_dev(v) for k, v in d.items()}
        t["Y"], t["dX"], t["dW"] = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl), gu.empty_dev(Kl, Nl)
        keep.append((d, t))
        p = axo.Problem.make(L.grid, (0, 0, 0), L.T, L.K, L.N)
        objs.append(axo.Layer(p, L.epilogue, 0, t["X"].data_ptr(), Kl, t["W"].data_ptr(), Nl,
                              t["bias"].data_ptr() if L.epilogue else None, t["Y"].data_ptr(), Nl,
                              t["dY"].data_ptr(), Nl, t["dX"].data_ptr(), Kl, t["dW"].data_ptr(), Nl))
    nws = axo.axo_layer_step_workspace_bytes(objs)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda:0")
    step(objs, ws.data_ptr(), nws, gu.stream())
    torch.cuda.synchronize()
    return keep


def check_sampled(L, d, t, seed, all_rows=False):
    M, Kl, Nl = L.shard
    rows = np.arange(M) if all_rows else syn.sample_rows_banded(M, 256, 16, seed)
    krows = np.arange(Kl) if all_rows else syn.sample_rows_banded(Kl, 256, 16, seed + 1)
    Y, dX, dW = gu.to_host(t["Y"]), gu.to_host(t["dX"]), gu.to_host(t["dW"])
    bias = d["bias"] if L.epilogue else None
    gu.assert_close(oracle, Y[rows], oracle.fc_fwd(d["X"], d["W"], bias, L.epilogue, rows=rows), L.name + " fwd")
    gu.assert_close(oracle, dX[rows], oracle.fc_dgrad(d["dY"], d["W"], rows=rows), L.name + " dgrad")
    gu.assert_close(oracle, dW[krows], oracle.fc_wgrad(d["X"], d["dY"], rows=krows), L.name + " wgrad")
    # nothing was left unwritten (the outputs were pre-filled with a NaN pattern)
    for a in (Y, dX, dW):
        assert not ((a & 0x7F80) == 0x7F80).any()


@pytest.mark.parametrize("cfg", ["cfg2", "cfg3", "cfg4"])
def test_full_size_single_layer(cfg):
    layers = syn.configs()[cfg]
    (d, t), = run_chain(layers)
    check_sampled(layers[0], d, t, 17, all_rows=True)


def test_full_size_chain_cfg5():
    layers = syn.configs()["cfg5"]
    keep = run_chain(layers)
    for L, (d, t) in zip(layers, keep):
        check_sampled(L, d, t, 23 + L.layer_index, all_rows=True)


def test_chain_equals_single_calls():
    """axo_layer_step must produce bit-identical results to the three entry points called one by one."""
    layers = syn.configs()["cfg5"][:2]
    keep = run_chain(layers)
    for L, (d, t) in zip(layers, keep):
        M, Kl, Nl = L.shard
        p = axo.Problem.make(L.grid, (0, 0, 0), L.T, L.K, L.N)
        Y, dX, dW = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl), gu.empty_dev(Kl, Nl)
        k = [gu.run_fwd(p, t["X"], t["W"], Y, t["bias"] if L.epilogue else None, L.epilogue),
             gu.run_dgrad(p, t["dY"], t["W"], dX), gu.run_wgrad(p, t["X"], t["dY"], dW)]
        torch.cuda.synchronize()
        assert torch.equal(Y, t["Y"]) and torch.equal(dX, t["dX"]) and torch.equal(dW, t["dW"])


def test_ordered_chain_cfg5_against_oracle():
    """The 12 products of the chain one launch each, in program order, sampled rows against the oracle."""
    layers = syn.configs()["cfg5"]
    keep = run_chain(layers, axo.axo_layer_step_ordered)
    for L, (d, t) in zip(layers, keep):
        check_sampled(L, d, t, 31 + L.layer_index)


@pytest.mark.parametrize("cfg", ["cfg2", "cfg5", "gpt20b"])
def test_scheduled_equals_ordered(cfg):
    """axo_layer_step finds these chains free of dependences and runs all their products in grouped
    launches, which cut the outputs into other tiles; every element is still reduced in the same
    order by the same instructions: bit-identical to one launch per product in program order."""
    layers = syn.configs()[cfg]
    a = run_chain(layers)
    b = run_chain(layers, axo.axo_layer_step_ordered)
    for (_, ta), (_, tb) in zip(a, b):
        for k in ("Y", "dX", "dW"):
            assert torch.equal(ta[k], tb[k]), k


def test_running_example_gpt20b():
    """The (2,2,4) shards of the paper's GPT-20B running example (Section 4) through axo_layer_step."""
    layers = syn.configs()["gpt20b"]
    keep = run_chain(layers)
    for L, (d, t) in zip(layers, keep):
        check_sampled(L, d, t, 41 + L.layer_index)
