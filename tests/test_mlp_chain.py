"""Two FC layers in a row on a 3D grid (paper Section 3.2, "Parallelizing an entire network"):
the block of O a GPU holds after the first layer is the block of I the second layer needs when
the second layer swaps the roles of the X and Y groups ("transposed" weights), so no data moves
between the layers.  Oracle-level check (no GPU): shard-by-shard simulation of
up -> (sum over the K-axis, bias, GELU) -> down against the unsharded computation."""
import numpy as np
import pytest

import axo_synth as syn
import oracle

GRIDS = [(2, 2, 2), (1, 2, 2), (2, 1, 1), (3, 2, 1)]


def mlp_inputs(T, K, N1, N2, seed):
    return (syn.normal_bf16(seed, 0, (T, K), 1.0), syn.normal_bf16(seed, 1, (K, N1), 0.05),
            syn.normal_bf16(seed, 2, (1, N1), 0.5)[0], syn.normal_bf16(seed, 3, (N1, N2), 0.05))


def gelu_tanh_f64(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def to_bf16_bits(a64):
    return syn.f32_to_bf16_bits(a64.astype(np.float32))


def coords(grid):
    gx, gy, gz = grid
    return [(ix, iy, iz) for iz in range(gz) for iy in range(gy) for ix in range(gx)]


@pytest.mark.parametrize("grid", GRIDS)
def test_output_layout_of_layer_one_is_input_layout_of_transposed_layer_two(grid):
    T, K, N1, N2 = 24, 36, 48, 12
    for c in coords(grid):
        rt1, _, rn1 = oracle.shard_slices(T, K, N1, grid, c, transposed=False)
        rt2, rk2, _ = oracle.shard_slices(T, N1, N2, grid, c, transposed=True)
        assert (rt1, rn1) == (rt2, rk2)
    # without the swap the blocks do not line up (on any grid where the X and Y coordinates can differ)
    gx, gy, _ = grid
    if gx > 1 or gy > 1:
        mismatch = [c for c in coords(grid)
                    if oracle.shard_slices(T, K, N1, grid, c, False)[2] != oracle.shard_slices(T, N1, N2, grid, c, False)[1]]
        assert mismatch


@pytest.mark.parametrize("grid", GRIDS)
def test_two_layer_chain_sharded_equals_unsharded(grid):
    T, K, N1, N2 = 48, 72, 96, 60
    X, W1, b1, W2 = mlp_inputs(T, K, N1, N2, 77)
    H_ref = oracle.fc_fwd(X, W1, b1, oracle.EPI_BIAS_GELU_TANH)
    H_bits = to_bf16_bits(H_ref)                      # the activation is stored in bf16 between the layers
    O_ref = oracle.fc_fwd(H_bits, W2)

    # layer one, default mapping: K over X, N over Y; all-reduce over X, then bias and GELU
    pre = np.zeros((T, N1))
    for c in coords(grid):
        rt, rk, rn = oracle.shard_slices(T, K, N1, grid, c, False)
        pre[rt, rn] += oracle.fc_fwd(X[rt, rk], W1[rk, rn])
    H = gelu_tanh_f64(pre + syn.bf16_bits_to_f64(b1)[None, :])
    assert np.allclose(H, H_ref, rtol=1e-11, atol=1e-13)
    # layer two, roles of X and Y swapped: K over Y, N over X; all-reduce over Y
    O = np.zeros((T, N2))
    for c in coords(grid):
        rt, rk, rn = oracle.shard_slices(T, N1, N2, grid, c, True)
        O[rt, rn] += oracle.fc_fwd(H_bits[rt, rk], W2[rk, rn])
    assert np.allclose(O, O_ref, rtol=1e-11, atol=1e-13)
