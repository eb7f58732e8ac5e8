"""GPU version of the two-layer chain (paper Section 3.2, "Parallelizing an entire network"): every
GPU of the grid is played in turn by the one device, all shards addressed IN PLACE inside the
global device tensors.  Layer one uses the default mapping, layer two the transposed one, and
the activation block a "GPU" writes is read by the same "GPU" in layer two without any copy or
re-layout.  The collectives (sum over the K-axis) and, where the K-axis is split, the bias and
GELU that must follow the sum are test-side torch code: they are not part of the library.

Tolerance: the final output has gone through three independent bf16 roundings (layer-one
partials, the stored activation, layer-two partials), each 1.66e-3 RMS, so about 2.9e-3 relative
Frobenius error is expected; bound 5e-3, and 2e-2 of the row maximum per element."""
import numpy as np
import pytest

import axo_synth as syn
import oracle
import paper_2305_13525_amd as axo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import gpu_util as gu  # noqa: E402

from test_mlp_chain import coords, mlp_inputs, to_bf16_bits  # noqa: E402

CHAIN_FRO_TOL, CHAIN_ELEM_TOL = 5e-3, 2e-2


def as_f32(t):
    return t.view(torch.bfloat16).float()


@pytest.mark.parametrize("grid,dims", [((2, 2, 2), (512, 512, 1024, 512)), ((1, 2, 2), (512, 256, 1024, 512)),
                                       ((2, 2, 2), (260, 144, 272, 80)), ((4, 2, 1), (256, 1024, 512, 1024))])
def test_two_layer_chain_in_place(grid, dims):
    T, K, N1, N2 = dims
    gx, gy, gz = grid
    Xb, W1b, b1b, W2b = mlp_inputs(T, K, N1, N2, 501)
    H_ref = oracle.fc_fwd(Xb, W1b, b1b, oracle.EPI_BIAS_GELU_TANH)
    O_ref = oracle.fc_fwd(to_bf16_bits(H_ref), W2b)

    X, W1, b1, W2 = gu.to_dev(Xb), gu.to_dev(W1b), gu.to_dev(b1b), gu.to_dev(W2b)
    H = gu.empty_dev(T, N1)                      # the activation, one global buffer: block (iz, iy) is what
    fused = gx == 1                              # the GPUs g_{*,iy,iz} hold after layer one
    pre = torch.zeros((T, N1), dtype=torch.float32, device="cuda:0")
    for c in coords(grid):
        p = axo.Problem.make(grid, c, T, K, N1, 0)
        _, (M, Kl, Nl, r0, k0, n0) = axo.axo_shard_dims(p)
        Xs, Ws = X[r0:r0 + M, k0:k0 + Kl], W1[k0:k0 + Kl, n0:n0 + Nl]
        if fused:   # K is not split: the epilogue is the layer's activation, written in place
            gu.run_fwd(p, Xs, Ws, H[r0:r0 + M, n0:n0 + Nl], b1[n0:n0 + Nl], axo.AXO_EPI_BIAS_GELU_TANH)
        else:
            part = gu.empty_dev(M, Nl)
            gu.run_fwd(p, Xs, Ws, part)
            pre[r0:r0 + M, n0:n0 + Nl] += as_f32(part)      # stands for the all-reduce over the K-axis
    if not fused:
        act = torch.nn.functional.gelu(pre + as_f32(b1)[None, :], approximate="tanh")
        H.copy_(act.to(torch.bfloat16).view(torch.int16))
    torch.cuda.synchronize()
    gu.assert_close(oracle, gu.to_host(H), H_ref, "activation", fro=CHAIN_FRO_TOL, per_elem=CHAIN_ELEM_TOL)

    O = torch.zeros((T, N2), dtype=torch.float32, device="cuda:0")
    for c in coords(grid):
        p1 = axo.Problem.make(grid, c, T, K, N1, 0)
        p2 = axo.Problem.make(grid, c, T, N1, N2, 1)
        _, (M1, _, Nl1, r01, _, n01) = axo.axo_shard_dims(p1)
        _, (M, Kl, Nl, r0, k0, n0) = axo.axo_shard_dims(p2)
        # the block this GPU produced in layer one is the block it consumes in layer two
        assert (M, Kl, r0, k0) == (M1, Nl1, r01, n01)
        part = gu.empty_dev(M, Nl)
        gu.run_fwd(p2, H[r0:r0 + M, k0:k0 + Kl], W2[k0:k0 + Kl, n0:n0 + Nl], part)
        O[r0:r0 + M, n0:n0 + Nl] += as_f32(part)            # all-reduce over the (now Y) K-axis
    torch.cuda.synchronize()
    got = O.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(got - O_ref) / np.linalg.norm(O_ref)
    assert rel <= CHAIN_FRO_TOL, rel
    assert np.all(np.abs(got - O_ref) <= CHAIN_ELEM_TOL * np.max(np.abs(O_ref), axis=1, keepdims=True))
