"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded bf16 inputs.  Tolerances: relative Frobenius error <= 2e-3 and every element within
1e-2 of its oracle row's infinity norm (gpu_util.REL_FRO_TOL / PER_ELEM_TOL).  Structured
inputs whose products are exactly representable must match bit for bit."""
import numpy as np
import pytest

import axo_synth as syn
import oracle
import paper_2305_13525_amd as axo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import gpu_util as gu  # noqa: E402


def P(M, Kl, Nl, grid=(1, 1, 1), coord=(0, 0, 0), transposed=0):
    gx, gy, gz = grid
    gk, gn = (gy, gx) if transposed else (gx, gy)
    return axo.Problem.make(grid, coord, M * gz, Kl * gk, Nl * gn, transposed)


def rand_trio(M, Kl, Nl, seed):
    return (syn.normal_bf16(seed, 0, (M, Kl), 1.0), syn.normal_bf16(seed, 1, (Kl, Nl), 0.02),
            syn.normal_bf16(seed, 2, (M, Nl), 1.0))


def check_trio(p, Xb, Wb, dYb, tag):
    Y, dX, dW = gu.trio(p, Xb, Wb, dYb)
    gu.assert_close(oracle, Y, oracle.fc_fwd(Xb, Wb), tag + " fwd")
    gu.assert_close(oracle, dX, oracle.fc_dgrad(dYb, Wb), tag + " dgrad")
    gu.assert_close(oracle, dW, oracle.fc_wgrad(Xb, dYb), tag + " wgrad")
    return Y, dX, dW


def test_cfg1_unsharded_trio():
    L = syn.configs()["cfg1"][0]
    d = syn.layer_inputs(L)
    p = axo.Problem.make(L.grid, (0, 0, 0), L.T, L.K, L.N)
    check_trio(p, d["X"], d["W"], d["dY"], "cfg1")


def test_cfg1_grid222_all_shards_and_decomposition_identity():
    """All 8 shard trios, serially, addressed in place inside the global device tensors (leading
    dimension > row length); each against the oracle's shard product, and the combined result
    (sum over the K-axis, N-axis, Z-axis respectively) against the unsharded oracle product."""
    L = syn.configs()["cfg1_grid222"][0]
    g = syn.global_inputs(L)
    Xg, Wg, dYg = gu.to_dev(g["X"]), gu.to_dev(g["W"]), gu.to_dev(g["dY"])
    Ysum = np.zeros((L.T, L.N))
    dXsum = np.zeros((L.T, L.K))
    dWsum = np.zeros((L.K, L.N))
    for iz in range(2):
        for iy in range(2):
            for ix in range(2):
                p = axo.Problem.make(L.grid, (ix, iy, iz), L.T, L.K, L.N)
                _, (M, Kl, Nl, r0, k0, n0) = axo.axo_shard_dims(p)
                Xs, Ws, dYs = Xg[r0:r0 + M, k0:k0 + Kl], Wg[k0:k0 + Kl, n0:n0 + Nl], dYg[r0:r0 + M, n0:n0 + Nl]
                Y, dX, dW = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl), gu.empty_dev(Kl, Nl)
                gu.run_fwd(p, Xs, Ws, Y)
                gu.run_dgrad(p, dYs, Ws, dX)
                gu.run_wgrad(p, Xs, dYs, dW)
                torch.cuda.synchronize()
                Xb, Wb, dYb = oracle.shards(g["X"], g["W"], g["dY"], L.grid, (ix, iy, iz))
                tag = f"shard {ix}{iy}{iz}"
                gu.assert_close(oracle, gu.to_host(Y), oracle.fc_fwd(Xb, Wb), tag + " fwd")
                gu.assert_close(oracle, gu.to_host(dX), oracle.fc_dgrad(dYb, Wb), tag + " dgrad")
                gu.assert_close(oracle, gu.to_host(dW), oracle.fc_wgrad(Xb, dYb), tag + " wgrad")
                Ysum[r0:r0 + M, n0:n0 + Nl] += syn.bf16_bits_to_f64(gu.to_host(Y))
                dXsum[r0:r0 + M, k0:k0 + Kl] += syn.bf16_bits_to_f64(gu.to_host(dX))
                dWsum[k0:k0 + Kl, n0:n0 + Nl] += syn.bf16_bits_to_f64(gu.to_host(dW))
    for got, ref, tag in ((Ysum, oracle.fc_fwd(g["X"], g["W"]), "Y"), (dXsum, oracle.fc_dgrad(g["dY"], g["W"]), "dX"),
                          (dWsum, oracle.fc_wgrad(g["X"], g["dY"]), "dW")):
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert rel <= gu.REL_FRO_TOL, (tag, rel)
        assert np.all(np.abs(got - ref) <= gu.PER_ELEM_TOL * np.max(np.abs(ref), axis=1, keepdims=True)), tag


RAGGED = [(1, 8, 8), (1000, 520, 264), (130, 40, 72), (257, 264, 136), (77, 1000, 48), (45, 100, 52),
          (129, 33, 127), (5, 7, 3), (256, 64, 256), (300, 1, 9), (128, 128, 128), (384, 96, 640),
          # outputs that miss the tuned kernel's granularity while the reduction fits it: the library
          # cuts these into a tuned interior and general-kernel strips (fwd; dgrad; wgrad; one strip only)
          (300, 128, 136), (520, 384, 264), (520, 264, 384), (384, 264, 136), (256, 128, 200), (260, 128, 128),
          (1030, 512, 1160),
          # token counts (the reduction of wgrad) of any length, odd ones included: the wgrad kernel
          # rounds the reduction up itself and reads the surplus rows as zeros
          (1000, 256, 384), (77, 256, 128), (1, 256, 128), (129, 512, 256), (4101, 256, 640), (300, 264, 136),
          # reductions of forward (Kl) and dgrad (Nl) that are multiples of 8 but not of 128, on tile-multiple
          # outputs and on ragged ones: the tuned kernel walks them rounded up and zeroes the surplus in LDS
          (256, 200, 128), (256, 128, 200), (512, 328, 392), (256, 8, 136), (256, 136, 8), (512, 1928, 256),
          (256, 256, 1928), (768, 2000, 520), (1000, 72, 1016), (256, 64, 120), (256, 192, 448)]


@pytest.mark.parametrize("M,Kl,Nl", RAGGED)
def test_ragged_and_tile_edge_shapes(M, Kl, Nl):
    """Shapes that are not multiples of any tile, with padded leading dimensions where the row
    length is not a multiple of 8."""
    Xb, Wb, dYb = rand_trio(M, Kl, Nl, 100 + M)
    pad = lambda n: (n + 7) // 8 * 8 + 8
    X = torch.zeros((M, pad(Kl)), dtype=torch.int16, device="cuda:0")
    W = torch.zeros((Kl, pad(Nl)), dtype=torch.int16, device="cuda:0")
    dY = torch.zeros((M, pad(Nl)), dtype=torch.int16, device="cuda:0")
    X[:, :Kl], W[:, :Nl], dY[:, :Nl] = gu.to_dev(Xb), gu.to_dev(Wb), gu.to_dev(dYb)
    Y, dX, dW = gu.empty_dev(M, pad(Nl)), gu.empty_dev(M, pad(Kl)), gu.empty_dev(Kl, pad(Nl))
    p = P(M, Kl, Nl)
    gu.run_fwd(p, X[:, :Kl], W[:, :Nl], Y[:, :Nl])
    gu.run_dgrad(p, dY[:, :Nl], W[:, :Nl], dX[:, :Kl])
    gu.run_wgrad(p, X[:, :Kl], dY[:, :Nl], dW[:, :Nl])
    torch.cuda.synchronize()
    Yh, dXh, dWh = gu.to_host(Y), gu.to_host(dX), gu.to_host(dW)
    gu.assert_close(oracle, Yh[:, :Nl], oracle.fc_fwd(Xb, Wb), "fwd")
    gu.assert_close(oracle, dXh[:, :Kl], oracle.fc_dgrad(dYb, Wb), "dgrad")
    gu.assert_close(oracle, dWh[:, :Nl], oracle.fc_wgrad(Xb, dYb), "wgrad")
    # nothing outside the logical matrix was written (the pad keeps its NaN fill)
    assert (Yh[:, Nl:] == 0x7FC0).all() and (dXh[:, Kl:] == 0x7FC0).all() and (dWh[:, Nl:] == 0x7FC0).all()


def test_reduction_tails_ignore_what_lies_behind_them():
    """Forward and dgrad with reductions that end inside the tuned kernel's last steps (2000 and 1928:
    16 resp. 8 real elements in the last but one step of 64, none in the last).  The shards sit in place
    inside wider buffers whose neighbouring columns and rows hold NaNs and infinities: what the kernel
    walks beyond the end of the reduction must not reach the result (a zero times a stray infinity would
    put a NaN into a row that has none), bit for bit the result of clean, contiguous operands."""
    for (M, Kl, Nl) in ((512, 2000, 256), (256, 256, 1928), (512, 328, 392)):
        Xb, Wb, dYb = rand_trio(M, Kl, Nl, 300 + Kl)
        p = P(M, Kl, Nl)
        poison = np.array([0x7FC0, 0x7F80, 0xFF80, 0x7FC1], dtype=np.uint16)

        def inside(bits, rows, cols):
            """bits in the top-left corner of a [rows, cols] buffer filled with NaN / inf patterns"""
            big = np.tile(poison, (rows * cols + 3) // 4)[:rows * cols].reshape(rows, cols).copy()
            big[:bits.shape[0], :bits.shape[1]] = bits
            return gu.to_dev(big)

        Xw, Ww, dYw = inside(Xb, M + 8, Kl + 136), inside(Wb, Kl + 136, Nl + 136), inside(dYb, M + 8, Nl + 136)
        Xs, Ws, dYs = Xw[:M, :Kl], Ww[:Kl, :Nl], dYw[:M, :Nl]
        assert axo.axo_fc_route(p, axo.AXO_OP_FWD, gu.ld(Xs), gu.ld(Ws), Nl)[1] in (axo.AXO_ROUTE_TILED, axo.AXO_ROUTE_COVERED)
        assert axo.axo_fc_route(p, axo.AXO_OP_DGRAD, gu.ld(dYs), gu.ld(Ws), Kl)[1] in (axo.AXO_ROUTE_TILED, axo.AXO_ROUTE_COVERED)
        Y, dX, dW = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl), gu.empty_dev(Kl, Nl)
        keep = [gu.run_fwd(p, Xs, Ws, Y), gu.run_dgrad(p, dYs, Ws, dX), gu.run_wgrad(p, Xs, dYs, dW)]
        torch.cuda.synchronize()
        del keep
        Yc, dXc, dWc = gu.trio(p, Xb, Wb, dYb)       # the same products on clean, contiguous operands
        for name, got, clean, ref in (("fwd", Y, Yc, oracle.fc_fwd(Xb, Wb)), ("dgrad", dX, dXc, oracle.fc_dgrad(dYb, Wb)),
                                      ("wgrad", dW, dWc, oracle.fc_wgrad(Xb, dYb))):
            got = gu.to_host(got)
            gu.assert_close(oracle, got, ref, f"{name} {(M, Kl, Nl)} inside poisoned buffers")
            assert np.array_equal(got, clean), name


def test_seeded_random_shapes_against_oracle():
    """Twenty-four seeded shapes with row lengths that are multiples of 8 (what the tuned kernel asks for),
    drawn so that every route occurs: whole tiles, covered outputs, reductions with tails, and the general
    kernel for the small ones.  Every element of all three products against the oracle."""
    rng = np.random.default_rng(20240)
    routes = set()
    for case in range(24):
        M = int(rng.choice([rng.integers(1, 300), rng.integers(256, 1100), 256 * rng.integers(1, 5)]))
        Kl = int(rng.choice([8 * rng.integers(1, 160), 128 * rng.integers(1, 10)]))
        Nl = int(rng.choice([8 * rng.integers(1, 160), 128 * rng.integers(1, 10)]))
        p = P(M, Kl, Nl)
        routes |= {axo.axo_fc_route(p, op, *lds)[1] for op, lds in
                   ((axo.AXO_OP_FWD, (Kl, Nl, Nl)), (axo.AXO_OP_DGRAD, (Nl, Nl, Kl)), (axo.AXO_OP_WGRAD, (Kl, Nl, Nl)))}
        Xb, Wb, dYb = rand_trio(M, Kl, Nl, 5000 + case)
        check_trio(p, Xb, Wb, dYb, f"case {case}: {(M, Kl, Nl)}")
    assert {axo.AXO_ROUTE_TILED, axo.AXO_ROUTE_COVERED, axo.AXO_ROUTE_GENERAL} <= routes


def test_empty_dimensions():
    # Kl == 0: forward of an empty sum is zero (then the epilogue); dW is empty
    Xb, Wb, dYb = rand_trio(16, 8, 24, 1)
    X, W, dY = gu.to_dev(Xb), gu.to_dev(Wb), gu.to_dev(dYb)
    bias_b = syn.normal_bf16(1, 3, (1, 24), 0.5)[0]
    bias = gu.to_dev(bias_b)
    p = P(16, 0, 24)
    Y = gu.empty_dev(16, 24)
    gu.run_fwd(p, X[:, :0], W[:0, :], Y)
    torch.cuda.synchronize()
    assert not gu.to_host(Y).any()
    gu.run_fwd(p, X[:, :0], W[:0, :], Y, bias, axo.AXO_EPI_BIAS)
    torch.cuda.synchronize()
    assert np.array_equal(gu.to_host(Y), np.tile(bias_b, (16, 1)))
    # M == 0: dW of an empty sum is zero
    p = P(0, 8, 24)
    dW = gu.empty_dev(8, 24)
    gu.run_wgrad(p, X[:0], dY[:0], dW)
    torch.cuda.synchronize()
    assert not gu.to_host(dW).any()
    # Nl == 0: dX of an empty sum is zero
    p = P(16, 8, 0)
    dX = gu.empty_dev(16, 8)
    gu.run_dgrad(p, dY[:, :0], W[:, :0], dX)
    torch.cuda.synchronize()
    assert not gu.to_host(dX).any()


@pytest.mark.parametrize("epi", [axo.AXO_EPI_BIAS, axo.AXO_EPI_BIAS_GELU_TANH, axo.AXO_EPI_BIAS_GELU_ERF])
@pytest.mark.parametrize("shape", [(200, 136, 264), (512, 256, 512), (520, 256, 392),   # the third: a covered output
                                   (512, 200, 256), (768, 1928, 392)])                  # reductions with a tail
def test_forward_epilogues(epi, shape):
    M, Kl, Nl = shape
    Xb = syn.normal_bf16(5, 0, (M, Kl), 1.0)
    Wb = syn.normal_bf16(5, 1, (Kl, Nl), 0.1)   # pre-activations of order 1: exercises the GELU knee
    bias_b = syn.normal_bf16(5, 3, (1, Nl), 0.5)[0]
    X, W, bias = gu.to_dev(Xb), gu.to_dev(Wb), gu.to_dev(bias_b)
    Y = gu.empty_dev(M, Nl)
    gu.run_fwd(P(M, Kl, Nl), X, W, Y, bias, epi)
    torch.cuda.synchronize()
    gu.assert_close(oracle, gu.to_host(Y), oracle.fc_fwd(Xb, Wb, bias_b, epi), f"epi {epi}")


def test_bias_only_at_k_coordinate_zero():
    """On a grid whose K-splitting axis has size 2 the bias is added on coordinate 0 only, so the
    two partial products sum to X.W + b (decomposition identity with bias)."""
    M, K, N = 64, 128, 96
    Xb, Wb = syn.normal_bf16(6, 0, (M, K), 1.0), syn.normal_bf16(6, 1, (K, N), 0.05)
    bias_b = syn.normal_bf16(6, 3, (1, N), 0.5)[0]
    Xg, Wg, bias = gu.to_dev(Xb), gu.to_dev(Wb), gu.to_dev(bias_b)
    total = np.zeros((M, N))
    zero_bias = np.zeros(N, dtype=np.uint16)
    for ix in range(2):
        p = axo.Problem.make((2, 1, 1), (ix, 0, 0), M, K, N)
        Y = gu.empty_dev(M, N)
        gu.run_fwd(p, Xg[:, ix * 64:(ix + 1) * 64], Wg[ix * 64:(ix + 1) * 64], Y, bias, axo.AXO_EPI_BIAS)
        torch.cuda.synchronize()
        ref = oracle.fc_fwd(Xb[:, ix * 64:(ix + 1) * 64], Wb[ix * 64:(ix + 1) * 64], bias_b if ix == 0 else zero_bias,
                            oracle.EPI_BIAS)
        gu.assert_close(oracle, gu.to_host(Y), ref, f"bias shard {ix}")
        total += syn.bf16_bits_to_f64(gu.to_host(Y))
    ref = oracle.fc_fwd(Xb, Wb, bias_b, oracle.EPI_BIAS)
    assert np.linalg.norm(total - ref) <= gu.REL_FRO_TOL * np.linalg.norm(ref)
    # transposed mapping: K is split over Gy, so iy decides
    for iy in range(2):
        p = axo.Problem.make((1, 2, 1), (0, iy, 0), M, K, N, 1)
        Y = gu.empty_dev(M, N)
        gu.run_fwd(p, Xg[:, iy * 64:(iy + 1) * 64], Wg[iy * 64:(iy + 1) * 64], Y, bias, axo.AXO_EPI_BIAS)
        torch.cuda.synchronize()
        ref = oracle.fc_fwd(Xb[:, iy * 64:(iy + 1) * 64], Wb[iy * 64:(iy + 1) * 64], bias_b if iy == 0 else zero_bias,
                            oracle.EPI_BIAS)
        gu.assert_close(oracle, gu.to_host(Y), ref, f"transposed bias shard {iy}")


@pytest.mark.parametrize("n", [64, 256, 520])
def test_structured_inputs_are_bit_exact(n):
    one = np.uint16(0x3F80)
    Xb = syn.normal_bf16(8, 0, (n + 40, n), 1.0)
    eye = np.zeros((n, n), dtype=np.uint16)
    eye[np.arange(n), np.arange(n)] = one
    p = P(n + 40, n, n)
    Y, dX, dW = gu.trio(p, Xb, eye, Xb)
    assert np.array_equal(Y, Xb), "X . I must reproduce X bit for bit"
    assert np.array_equal(dX, Xb), "dY . I^T must reproduce dY bit for bit"
    # one-hot X row: forward picks (a power-of-two multiple of) one row of W
    Wb = syn.normal_bf16(8, 1, (n, n), 0.02)
    hot = np.zeros((n + 40, n), dtype=np.uint16)
    hot[n + 39, n - 1] = np.uint16(0x4000)  # 2.0 in the last row / last column
    hot[0, 0] = np.uint16(0x3F00)           # 0.5
    Y, _, dW = gu.trio(p, hot, Wb, Xb)
    assert np.array_equal(syn.bf16_bits_to_f64(Y[n + 39]), 2.0 * syn.bf16_bits_to_f64(Wb[n - 1]))
    assert np.array_equal(syn.bf16_bits_to_f64(Y[0]), 0.5 * syn.bf16_bits_to_f64(Wb[0]))
    assert not syn.bf16_bits_to_f64(Y[1:n + 39]).any()
    # wgrad of the one-hot X: row n-1 of dW is 2 * dY[last], row 0 is 0.5 * dY[0], the rest zero
    assert np.array_equal(syn.bf16_bits_to_f64(dW[n - 1]), 2.0 * syn.bf16_bits_to_f64(Xb[n + 39]))
    assert np.array_equal(syn.bf16_bits_to_f64(dW[0]), 0.5 * syn.bf16_bits_to_f64(Xb[0]))
    assert not syn.bf16_bits_to_f64(dW[1:n - 1]).any()


TILED = [(512, 192, 768), (256, 64, 512), (768, 448, 256), (1024, 128, 1280), (256, 2048, 256),
         (256, 64, 128), (512, 128, 384), (768, 256, 640), (256, 512, 896), (1280, 384, 1152)]


@pytest.mark.parametrize("M,Kl,Nl", TILED)
def test_tile_multiple_shapes(M, Kl, Nl):
    """Shapes that are whole multiples of the tuned kernel's tile in all three roles, several tiles
    wide and high, with different extents per dimension so that a swapped index cannot cancel."""
    Xb, Wb, dYb = rand_trio(M, Kl, Nl, 200 + Kl)
    check_trio(P(M, Kl, Nl), Xb, Wb, dYb, f"tiled {M}x{Kl}x{Nl}")


def test_tile_multiple_shapes_in_place_and_structured():
    """Tuned-kernel shapes addressed inside larger buffers (leading dimension > row length), and an
    identity weight that must reproduce the activation bit for bit."""
    M, Kl, Nl = 512, 256, 768
    Xb, Wb, dYb = rand_trio(M, Kl, Nl, 31)
    big = lambda r, c: torch.zeros((r, c + 64), dtype=torch.int16, device="cuda:0")
    X, W, dY = big(M, Kl), big(Kl, Nl), big(M, Nl)
    X[:, 8:8 + Kl], W[:, 16:16 + Nl], dY[:, 24:24 + Nl] = gu.to_dev(Xb), gu.to_dev(Wb), gu.to_dev(dYb)
    Y, dX, dW = gu.empty_dev(M, Nl + 64), gu.empty_dev(M, Kl + 64), gu.empty_dev(Kl, Nl + 64)
    p = P(M, Kl, Nl)
    gu.run_fwd(p, X[:, 8:8 + Kl], W[:, 16:16 + Nl], Y[:, 32:32 + Nl])
    gu.run_dgrad(p, dY[:, 24:24 + Nl], W[:, 16:16 + Nl], dX[:, 8:8 + Kl])
    gu.run_wgrad(p, X[:, 8:8 + Kl], dY[:, 24:24 + Nl], dW[:, 40:40 + Nl])
    torch.cuda.synchronize()
    Yh, dXh, dWh = gu.to_host(Y), gu.to_host(dX), gu.to_host(dW)
    gu.assert_close(oracle, Yh[:, 32:32 + Nl], oracle.fc_fwd(Xb, Wb), "fwd")
    gu.assert_close(oracle, dXh[:, 8:8 + Kl], oracle.fc_dgrad(dYb, Wb), "dgrad")
    gu.assert_close(oracle, dWh[:, 40:40 + Nl], oracle.fc_wgrad(Xb, dYb), "wgrad")
    assert (Yh[:, :32] == 0x7FC0).all() and (Yh[:, 32 + Nl:] == 0x7FC0).all()
    assert (dXh[:, :8] == 0x7FC0).all() and (dXh[:, 8 + Kl:] == 0x7FC0).all()
    assert (dWh[:, :40] == 0x7FC0).all() and (dWh[:, 40 + Nl:] == 0x7FC0).all()
    n = 512
    eye = np.zeros((n, n), dtype=np.uint16)
    eye[np.arange(n), np.arange(n)] = 0x3F80
    Xs = syn.normal_bf16(32, 0, (768, n), 1.0)
    Y2, dX2, dW2 = gu.trio(P(768, n, n), Xs, eye, Xs)
    assert np.array_equal(Y2, Xs) and np.array_equal(dX2, Xs)


def test_adjoint_identity_on_gpu_results():
    M, Kl, Nl = 384, 320, 448
    Xb, Wb, dYb = rand_trio(M, Kl, Nl, 9)
    Y, dX, dW = (syn.bf16_bits_to_f64(a) for a in gu.trio(P(M, Kl, Nl), Xb, Wb, dYb))
    Xf, Wf, Gf = (syn.bf16_bits_to_f64(a) for a in (Xb, Wb, dYb))
    a, b, c = np.sum(Gf * Y), np.sum(dX * Xf), np.sum(dW * Wf)
    scale = np.linalg.norm(Gf) * np.linalg.norm(Y)
    assert abs(a - b) <= 1e-3 * scale and abs(a - c) <= 1e-3 * scale


def test_results_are_reproducible_run_to_run():
    M, Kl, Nl = 512, 768, 256
    Xb, Wb, dYb = rand_trio(M, Kl, Nl, 10)
    r1 = gu.trio(P(M, Kl, Nl), Xb, Wb, dYb)
    r2 = gu.trio(P(M, Kl, Nl), Xb, Wb, dYb)
    for a, b in zip(r1, r2):
        assert np.array_equal(a, b)


def test_rounding_is_nearest_even():
    """Products chosen to land exactly on bf16 rounding ties: X row = [1, 2^-8], W col = [1, t]."""
    n = 64
    X = np.zeros((n, n), dtype=np.uint16)
    W = np.zeros((n, n), dtype=np.uint16)
    X[:, 0] = 0x3F80             # 1.0
    X[:, 1] = 0x3B80             # 2^-8
    W[0, :] = 0x3F80             # 1.0
    W[1, 0::4] = 0x3F80          # 1 + 2^-8  -> tie, rounds to even 1.0         (0x3F80)
    W[1, 1::4] = 0x4040          # 1 + 3*2^-8 -> rounds to nearest 1 + 2^-6 ... (checked against the oracle)
    W[1, 2::4] = 0x3FC0          # 1 + 1.5*2^-8
    W[1, 3::4] = 0x0000
    Y, _, _ = gu.trio(P(n, n, n), X, W, X)
    ref = oracle.fc_fwd(X, W)
    want = syn.f32_to_bf16_bits(ref.astype(np.float32))  # every sum here is exact in fp32
    assert np.array_equal(Y, want)
    assert Y[0, 0] == 0x3F80 and Y[0, 3] == 0x3F80


def test_grouped_step_mixed_shapes_against_oracle():
    """axo_layer_step on an independent chain that mixes shapes the tiled kernel takes, shapes it does not
    (ragged; a product with a 128-row output) and an empty layer: every element against the oracle."""
    shapes = [(256, 256, 256), (300, 72, 136), (256, 128, 384), (512, 384, 640), (0, 64, 64), (768, 256, 1152),
              (512, 328, 392), (256, 200, 1928)]   # reductions that end inside the tuned kernel's last steps
    layers, keep = [], []
    for i, (M, Kl, Nl) in enumerate(shapes):
        Xb, Wb, dYb = rand_trio(M, Kl, Nl, 900 + i)
        bias_b = syn.normal_bf16(900 + i, 3, (1, Nl), 0.5)[0]
        epi = axo.AXO_EPI_BIAS_GELU_TANH if i % 2 else axo.AXO_EPI_NONE
        t = dict(X=gu.to_dev(Xb), W=gu.to_dev(Wb), dY=gu.to_dev(dYb), bias=gu.to_dev(bias_b),
                 Y=gu.empty_dev(M, Nl), dX=gu.empty_dev(M, Kl), dW=gu.empty_dev(Kl, Nl))
        keep.append((Xb, Wb, dYb, bias_b, epi, t))
        layers.append(axo.Layer(P(M, Kl, Nl), epi, 0, t["X"].data_ptr(), Kl, t["W"].data_ptr(), Nl,
                                t["bias"].data_ptr() if epi else None, t["Y"].data_ptr(), Nl,
                                t["dY"].data_ptr(), Nl, t["dX"].data_ptr(), Kl, t["dW"].data_ptr(), Nl))
    assert axo.axo_layer_step_levels(layers)[1] == 1
    axo.axo_layer_step(layers, None, 0, gu.stream())
    torch.cuda.synchronize()
    for i, (Xb, Wb, dYb, bias_b, epi, t) in enumerate(keep):
        if Xb.shape[0] == 0:  # no tokens: dW is an empty sum
            assert not gu.to_host(t["dW"]).any()
            continue
        tag = f"layer {i}"
        gu.assert_close(oracle, gu.to_host(t["Y"]), oracle.fc_fwd(Xb, Wb, bias_b if epi else None, epi), tag + " fwd")
        gu.assert_close(oracle, gu.to_host(t["dX"]), oracle.fc_dgrad(dYb, Wb), tag + " dgrad")
        gu.assert_close(oracle, gu.to_host(t["dW"]), oracle.fc_wgrad(Xb, dYb), tag + " wgrad")


@pytest.mark.parametrize("step", ["axo_layer_step", "axo_layer_step_ordered"])
def test_step_with_dependent_layers(step):
    """A chain whose products depend on each other: layer one reads the Y that layer zero writes,
    and layer zero's dY is the dX that layer one writes.  axo_layer_step has to find the two
    dependence levels (fwd 0 and dgrad 1 first; then fwd 1, wgrad 1, dgrad 0, wgrad 0) and keep
    them apart.  The second product of each dependence is checked against the oracle applied to
    the bits the first one produced."""
    M, K0, N0, N1 = 512, 256, 512, 384
    Xb, W0b, _ = rand_trio(M, K0, N0, 950)
    _, W1b, dY1b = rand_trio(M, N0, N1, 951)
    X, W0, W1, dY1 = gu.to_dev(Xb), gu.to_dev(W0b), gu.to_dev(W1b), gu.to_dev(dY1b)
    Y0, Y1 = gu.empty_dev(M, N0), gu.empty_dev(M, N1)
    dX1, dX0 = gu.empty_dev(M, N0), gu.empty_dev(M, K0)
    dW0, dW1 = gu.empty_dev(K0, N0), gu.empty_dev(N0, N1)
    layers = [
        axo.Layer(P(M, K0, N0), 0, 0, X.data_ptr(), K0, W0.data_ptr(), N0, None, Y0.data_ptr(), N0,
                  dX1.data_ptr(), N0, dX0.data_ptr(), K0, dW0.data_ptr(), N0),
        axo.Layer(P(M, N0, N1), 0, 0, Y0.data_ptr(), N0, W1.data_ptr(), N1, None, Y1.data_ptr(), N1,
                  dY1.data_ptr(), N1, dX1.data_ptr(), N0, dW1.data_ptr(), N1),
    ]
    assert axo.axo_layer_step_levels(layers)[1:] == (2, [0, 1, 0, 1, 1, 1])
    getattr(axo, step)(layers, None, 0, gu.stream())
    torch.cuda.synchronize()
    Y0b, dX1b = gu.to_host(Y0), gu.to_host(dX1)
    gu.assert_close(oracle, Y0b, oracle.fc_fwd(Xb, W0b), "fwd 0")
    gu.assert_close(oracle, gu.to_host(Y1), oracle.fc_fwd(Y0b, W1b), "fwd 1 on fwd 0's output")
    gu.assert_close(oracle, dX1b, oracle.fc_dgrad(dY1b, W1b), "dgrad 1")
    gu.assert_close(oracle, gu.to_host(dW1), oracle.fc_wgrad(Y0b, dY1b), "wgrad 1 on fwd 0's output")
    gu.assert_close(oracle, gu.to_host(dX0), oracle.fc_dgrad(dX1b, W0b), "dgrad 0 on dgrad 1's output")
    gu.assert_close(oracle, gu.to_host(dW0), oracle.fc_wgrad(Xb, dX1b), "wgrad 0 on dgrad 1's output")


@pytest.mark.parametrize("ld_elems,what", [(4_300_000, "tiled kernel, byte offsets above 2^31"),
                                           (8_400_000, "span above 4 GiB: general kernel")])
def test_very_large_leading_dimensions(ld_elems, what):
    """The largest strides the library takes.  Every input is a 256-row slice of a buffer whose rows
    are ld_elems apart.  At 4.3 M elements the 256 rows a workgroup walks span 2.2 GB: the tiled
    kernel still takes them, with unsigned 32-bit byte offsets above 2^31.  At 8.4 M the span
    passes 4 GiB and the library has to route the product to the general kernel (64-bit indices)."""
    M = Kl = Nl = 256
    Xb, Wb, dYb = rand_trio(M, Kl, Nl, 970)
    held = []

    def wide(bits):
        big = torch.empty((bits.shape[0], ld_elems), dtype=torch.int16, device="cuda:0")
        held.append(big)
        view = big[:, :bits.shape[1]]
        view.copy_(gu.to_dev(bits))
        return view

    X, W, dY = wide(Xb), wide(Wb), wide(dYb)
    assert gu.ld(X) == ld_elems and X.data_ptr() % 16 == 0
    Y, dX, dW = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl), gu.empty_dev(Kl, Nl)
    p = P(M, Kl, Nl)
    keep = [gu.run_fwd(p, X, W, Y), gu.run_dgrad(p, dY, W, dX), gu.run_wgrad(p, X, dY, dW)]
    torch.cuda.synchronize()
    gu.assert_close(oracle, gu.to_host(Y), oracle.fc_fwd(Xb, Wb), what + " fwd")
    gu.assert_close(oracle, gu.to_host(dX), oracle.fc_dgrad(dYb, Wb), what + " dgrad")
    gu.assert_close(oracle, gu.to_host(dW), oracle.fc_wgrad(Xb, dYb), what + " wgrad")
    del keep, held, X, W, dY
    torch.cuda.empty_cache()


def test_wgrad_ragged_token_count_with_a_very_large_leading_dimension():
    """wgrad walks its token count rounded up to 128.  With 450 tokens 4.3 M elements apart the 450
    rows span 3.87 GB (below the tuned kernel's 4 GiB limit) but the 512 rows the kernel would walk do
    not: the library has to send the product to the general kernel."""
    M, Kl, Nl, ld_elems = 450, 256, 384, 4_300_000
    Xb, _, dYb = rand_trio(M, Kl, Nl, 971)
    p = P(M, Kl, Nl)
    assert axo.axo_fc_route(p, axo.AXO_OP_WGRAD, ld_elems, ld_elems, Nl)[1] == axo.AXO_ROUTE_GENERAL
    held = []

    def wide(bits):
        big = torch.empty((bits.shape[0], ld_elems), dtype=torch.int16, device="cuda:0")
        held.append(big)
        view = big[:, :bits.shape[1]]
        view.copy_(gu.to_dev(bits))
        return view

    X, dY, dW = wide(Xb), wide(dYb), gu.empty_dev(Kl, Nl)
    keep = gu.run_wgrad(p, X, dY, dW)
    torch.cuda.synchronize()
    gu.assert_close(oracle, gu.to_host(dW), oracle.fc_wgrad(Xb, dYb), "wgrad, 450 tokens 4.3 M elements apart")
    del keep, held, X, dY
    torch.cuda.empty_cache()


def test_concurrent_host_threads_on_their_own_streams():
    """Four host threads enqueue products of different shapes on their own streams at the same time
    (ctypes releases the interpreter lock during a call, so the library's planners and their
    per-shape caches are entered concurrently).  Every result is checked against the oracle."""
    import threading
    shapes = [(256, 256, 256), (512, 128, 384), (300, 72, 136), (768, 256, 640)]
    jobs, errors = [], []
    for i, (M, Kl, Nl) in enumerate(shapes):
        Xb, Wb, dYb = rand_trio(M, Kl, Nl, 980 + i)
        t = dict(X=gu.to_dev(Xb), W=gu.to_dev(Wb), dY=gu.to_dev(dYb), Y=gu.empty_dev(M, Nl), dX=gu.empty_dev(M, Kl),
                 dW=gu.empty_dev(Kl, Nl), stream=torch.cuda.Stream())
        jobs.append(((M, Kl, Nl), (Xb, Wb, dYb), t))
    torch.cuda.synchronize()

    def work(shape, t):
        try:
            M, Kl, Nl = shape
            p, st = P(M, Kl, Nl), t["stream"].cuda_stream
            for _ in range(20):
                axo.axo_fc_fwd(p, t["X"].data_ptr(), Kl, t["W"].data_ptr(), Nl, None, 0, t["Y"].data_ptr(), Nl,
                               None, 0, st)
                axo.axo_fc_dgrad(p, t["dY"].data_ptr(), Nl, t["W"].data_ptr(), Nl, t["dX"].data_ptr(), Kl, None, 0, st)
                axo.axo_fc_wgrad(p, t["X"].data_ptr(), Kl, t["dY"].data_ptr(), Nl, t["dW"].data_ptr(), Nl, None, 0, st)
        except Exception as e:  # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(shape, t)) for shape, _, t in jobs]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for shape, (Xb, Wb, dYb), t in jobs:
        tag = f"thread {shape}"
        gu.assert_close(oracle, gu.to_host(t["Y"]), oracle.fc_fwd(Xb, Wb), tag + " fwd")
        gu.assert_close(oracle, gu.to_host(t["dX"]), oracle.fc_dgrad(dYb, Wb), tag + " dgrad")
        gu.assert_close(oracle, gu.to_host(t["dW"]), oracle.fc_wgrad(Xb, dYb), tag + " wgrad")


def test_denormals_infinities_and_nans():
    """Values outside the benchmark's Gaussian inputs.  bf16 denormal inputs are honoured (not
    flushed: a row of 256 denormals times ones gives their exact sum); an infinity makes its row
    infinite, and NaN where it meets a zero; a NaN makes its whole row NaN; rows without special
    values are not disturbed.  The oracle computes the same classes in fp64."""
    M = Kl = Nl = 256
    Xb, Wb, _ = rand_trio(M, Kl, Nl, 990)
    Xb = Xb.copy()
    Wb = Wb.copy()
    Xb[0, :] = 0x0040          # 2^-127, a bf16 denormal
    Wb[:, 0] = 0x3F80          # a column of ones: Y[0, 0] = 256 * 2^-127 = 2^-119 exactly
    Xb[2, 5] = 0x7F80          # +infinity
    Wb[5, 2] = 0x0000          # times zero in column 2
    Xb[3, 7] = 0x7FC0          # NaN
    X, W, Y = gu.to_dev(Xb), gu.to_dev(Wb), gu.empty_dev(M, Nl)
    keep = gu.run_fwd(P(M, Kl, Nl), X, W, Y)
    torch.cuda.synchronize()
    del keep
    got = gu.to_host(Y)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.fc_fwd(Xb, Wb)
    gotf = syn.bf16_bits_to_f64(got)
    assert got[0, 0] == 0x0400 and ref[0, 0] == 2.0 ** -119
    finite_rows = np.array([r for r in range(M) if r not in (2, 3)])
    gu.assert_close(oracle, got[finite_rows], ref[finite_rows], "rows without special values")
    assert np.isnan(ref[2, 2]) and np.isnan(gotf[2, 2])                      # inf * 0
    inf_cols = np.isinf(ref[2])
    assert inf_cols.sum() == Nl - 1
    assert np.array_equal(np.isinf(gotf[2]), inf_cols) and np.array_equal(np.sign(gotf[2][inf_cols]), np.sign(ref[2][inf_cols]))
    assert np.isnan(ref[3]).all() and np.isnan(gotf[3]).all()


def check_value_classes(got_bits, ref, special_rows, what):
    """NaNs where the oracle has NaNs, infinities of the same sign where it has infinities, and the
    rows without special values within the usual tolerances."""
    gotf = syn.bf16_bits_to_f64(got_bits)
    assert np.array_equal(np.isnan(gotf), np.isnan(ref)), what
    assert np.array_equal(np.isinf(gotf), np.isinf(ref)), what
    inf = np.isinf(ref)
    assert np.array_equal(np.sign(gotf[inf]), np.sign(ref[inf])), what
    plain = np.array([r for r in range(ref.shape[0]) if r not in special_rows], dtype=np.int64)
    if plain.size:
        assert np.isfinite(ref[plain]).all()
        gu.assert_close(oracle, got_bits[plain], ref[plain], what)


def test_special_values_in_wgrad_with_a_ragged_token_count():
    """wgrad on the tuned kernel with a token count that is no multiple of 128: the kernel walks 1024
    rows of X and dY and must read rows 1000..1023 as zeros.  Here those rows EXIST in memory (the
    operands are the first 1000 rows of larger buffers) and hold NaNs, so a surplus row that leaked in
    would poison every output; an infinity sits in the last valid row, a NaN elsewhere."""
    M, Kl, Nl = 1000, 256, 384
    Xb, _, dYb = rand_trio(M, Kl, Nl, 991)
    Xb, dYb = Xb.copy(), dYb.copy()
    Xb[999, 5] = 0x7F80         # +inf in the last token: row 5 of dW becomes +-inf ...
    dYb[999, 17] = 0x0000       # ... and NaN where it meets a zero
    Xb[10, 7] = 0x7FC0          # NaN: row 7 of dW is NaN
    dYb[500, 40] = 0xFF80       # -inf in dY: column 40 of dW is +-inf (NaN in rows 5 and 7)
    Xfull = np.full((1024, Kl), 0x7FC0, dtype=np.uint16)
    dYfull = np.full((1024, Nl), 0x7FC0, dtype=np.uint16)
    Xfull[:M], dYfull[:M] = Xb, dYb
    X, dY, dW = gu.to_dev(Xfull), gu.to_dev(dYfull), gu.empty_dev(Kl, Nl)
    p = P(M, Kl, Nl)
    assert axo.axo_fc_route(p, axo.AXO_OP_WGRAD, Kl, Nl, Nl)[1] == axo.AXO_ROUTE_TILED
    keep = gu.run_wgrad(p, X, dY, dW)
    torch.cuda.synchronize()
    del keep
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.fc_wgrad(Xb, dYb)
    assert np.isnan(ref[7]).all() and np.isnan(ref[5, 17]) and np.isinf(ref[0, 40])
    got = gu.to_host(dW)
    cols = np.array([c for c in range(Nl) if c != 40])          # column 40 is special in every row
    check_value_classes(got[:, cols], ref[:, cols], (5, 7), "wgrad, ragged token count")
    check_value_classes(got[:, 40:41], ref[:, 40:41], range(Kl), "wgrad, ragged token count, column 40")


def test_special_values_in_an_output_covered_with_overlapping_tiles():
    """A forward product whose ragged output is covered with whole tiles that overlap: elements in the
    overlap are computed twice and must come out the same, special values included."""
    M, Kl, Nl = 520, 384, 264
    Xb, Wb, _ = rand_trio(M, Kl, Nl, 992)
    Xb, Wb = Xb.copy(), Wb.copy()
    Xb[519, 3] = 0x7F80         # +inf in the last row (inside the band of the last 256 rows only)
    Wb[3, 263] = 0x0000         # times zero in the last column (inside the band of the last 128 columns only)
    Xb[300, 9] = 0x7FC0         # NaN in a row that interior and row band both cover
    X, W, Y = gu.to_dev(Xb), gu.to_dev(Wb), gu.empty_dev(M, Nl)
    p = P(M, Kl, Nl)
    assert axo.axo_fc_route(p, axo.AXO_OP_FWD, Kl, Nl, Nl)[1] == axo.AXO_ROUTE_COVERED
    keep = gu.run_fwd(p, X, W, Y)
    torch.cuda.synchronize()
    del keep
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.fc_fwd(Xb, Wb)
    assert np.isnan(ref[519, 263]) and np.isnan(ref[300]).all()
    check_value_classes(gu.to_host(Y), ref, (300, 519), "covered forward")


def test_scheduled_step_equals_ordered_step_on_random_dependent_chains():
    """Seeded random chains whose buffers are drawn from a small pool of equally shaped matrices, so
    that products read what others write, overwrite what others read and write to the same place
    in many combinations.  axo_layer_step (dependence levels, grouped launches) must leave every
    buffer of the pool exactly as axo_layer_step_ordered (one launch per product, program order)
    does.  A dependence the analysis missed would let two products race and show up here."""
    import random
    D = 256                                    # M = Kl = Nl: every buffer can play every role
    p = P(D, D, D)
    rnd = random.Random(11)
    sigma = 1.0 / 16.0                         # keeps magnitudes stable through chained products
    n_levels_seen = set()
    for case in range(12):
        n = rnd.randint(2, 4)
        pool_bits = [syn.normal_bf16(1000 + case, k, (D, D), sigma) for k in range(rnd.randint(5, 4 * n))]
        choose = lambda banned=(): rnd.choice([i for i in range(len(pool_bits)) if i not in banned])
        roles = []
        for _ in range(n):
            X, W, dY = choose(), choose(), choose()
            Y = choose((X, W))                 # a product's output may not overlap its own inputs
            dX = choose((dY, W))
            dW = choose((X, dY))
            roles.append((X, W, Y, dY, dX, dW))
        results = []
        for step in (axo.axo_layer_step, axo.axo_layer_step_ordered):
            pool = [gu.to_dev(b) for b in pool_bits]
            layers = [axo.Layer(p, 0, 0, pool[X].data_ptr(), D, pool[W].data_ptr(), D, None, pool[Y].data_ptr(), D,
                                pool[dY].data_ptr(), D, pool[dX].data_ptr(), D, pool[dW].data_ptr(), D)
                      for X, W, Y, dY, dX, dW in roles]
            if step is axo.axo_layer_step:
                n_levels_seen.add(axo.axo_layer_step_levels(layers)[1])
            step(layers, None, 0, gu.stream())
            torch.cuda.synchronize()
            results.append(pool)
        for k, (a, b) in enumerate(zip(*results)):
            assert torch.equal(a, b), (case, k, roles)
    assert len(n_levels_seen) >= 3             # the cases really differ in their dependence structure
