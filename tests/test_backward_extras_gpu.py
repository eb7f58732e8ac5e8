"""GPU parity of the backward-side extras against the fp64 oracle: dgrad with the GELU derivative
fused in, wgrad accumulated into an fp32 matrix, and the bias gradient.  Same tolerances as the
products for the bf16 output; the fp32 outputs are held to fp32 summation error."""
import numpy as np
import pytest

import axo_synth as syn
import oracle
import paper_2305_13525_amd as axo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import gpu_util as gu  # noqa: E402

SHAPES = [(256, 256, 256), (512, 384, 640), (300, 72, 136), (1024, 128, 1280), (77, 40, 24), (768, 256, 1152),
          (520, 264, 384), (384, 264, 136),   # tuned interior plus strips or bands
          (1000, 256, 384),                   # wgrad on the tuned kernel with a reduction that is no multiple of 128
          (512, 256, 328), (768, 392, 1928)]  # dgrad (reduction Nl) with a tail on the tuned kernel


def P(M, Kl, Nl):
    return axo.Problem.make((1, 1, 1), (0, 0, 0), M, Kl, Nl)


@pytest.mark.parametrize("act", [axo.AXO_EPI_BIAS_GELU_TANH, axo.AXO_EPI_BIAS_GELU_ERF])
@pytest.mark.parametrize("M,Kl,Nl", SHAPES)
def test_dgrad_through_gelu(M, Kl, Nl, act):
    dYb, Wb = syn.normal_bf16(21, 0, (M, Nl), 1.0), syn.normal_bf16(21, 1, (Kl, Nl), 0.05)
    Pb = syn.normal_bf16(21, 2, (M, Kl), 1.5)      # pre-activations on both sides of the GELU's bend
    dY, W, pre, dX = gu.to_dev(dYb), gu.to_dev(Wb), gu.to_dev(Pb), gu.empty_dev(M, Kl)
    axo.axo_fc_dgrad_act(P(M, Kl, Nl), dY.data_ptr(), Nl, W.data_ptr(), Nl, pre.data_ptr(), Kl, act, dX.data_ptr(), Kl,
                         None, 0, gu.stream())
    torch.cuda.synchronize()
    gu.assert_close(oracle, gu.to_host(dX), oracle.fc_dgrad_act(dYb, Wb, Pb, act), f"dgrad_act {act}")


@pytest.mark.parametrize("act", [0, axo.AXO_EPI_BIAS_GELU_TANH, axo.AXO_EPI_BIAS_GELU_ERF])
@pytest.mark.parametrize("M,Kl,Nl", [(512, 512, 512),    # 256x256 tiles only
                                     (512, 128, 256),    # 256x128 tiles only
                                     (512, 640, 384)])   # both tile sizes in one launch
def test_dgrad_epilogues_by_position(M, Kl, Nl, act):
    """Every dgrad epilogue kind on both tile sizes, bit for bit and by position.  W holds one 1 per row
    (W[k, k % Nl] = 1), so dY . W^T puts dY[t, k % Nl] at [t, k] exactly; dY holds small integers that
    encode their position; the pre-activations are 0, +20 or -20, where both GELU derivatives are
    exactly 1/2, 1 and 0.  An output element that lands in the wrong place, or takes its factor from the
    wrong place, differs in its bits."""
    rng = np.random.default_rng(5)
    t, n = np.meshgrid(np.arange(M), np.arange(Nl), indexing="ij")
    dYv = ((t * 7 + n * 3) % 253 - 126).astype(np.float32)          # integers in [-126, 126]: exact in bf16
    Wv = np.zeros((Kl, Nl), dtype=np.float32)
    Wv[np.arange(Kl), np.arange(Kl) % Nl] = 1.0
    sel = rng.integers(0, 3, size=(M, Kl))
    prev = np.choose(sel, [0.0, 20.0, -20.0]).astype(np.float32)
    factor = np.choose(sel, [0.5, 1.0, 0.0]).astype(np.float32)
    dYb, Wb, Pb = syn.f32_to_bf16_bits(dYv), syn.f32_to_bf16_bits(Wv), syn.f32_to_bf16_bits(prev)
    want = dYv[:, np.arange(Kl) % Nl] * (factor if act else 1.0)    # halves of integers <= 126: exact in bf16
    dY, W, pre, dX = gu.to_dev(dYb), gu.to_dev(Wb), gu.to_dev(Pb), gu.empty_dev(M, Kl)
    if act:
        axo.axo_fc_dgrad_act(P(M, Kl, Nl), dY.data_ptr(), Nl, W.data_ptr(), Nl, pre.data_ptr(), Kl, act, dX.data_ptr(), Kl,
                             None, 0, gu.stream())
    else:
        axo.axo_fc_dgrad(P(M, Kl, Nl), dY.data_ptr(), Nl, W.data_ptr(), Nl, dX.data_ptr(), Kl, None, 0, gu.stream())
    torch.cuda.synchronize()
    got = syn.bf16_bits_to_f64(gu.to_host(dX))
    assert np.array_equal(got, want.astype(np.float64)), np.argwhere(got != want)[:5]   # -0 == 0 counts as equal
    # the oracle agrees with the construction (so the expectation is not this test's own invention)
    ref = oracle.fc_dgrad_act(dYb, Wb, Pb, act) if act else oracle.fc_dgrad(dYb, Wb)
    assert np.max(np.abs(ref - want)) <= 1e-12 * 126


def test_dgrad_through_gelu_in_place_shard():
    """Shard of a (2,2,2) grid addressed inside the global tensors (leading dimensions > row length)."""
    T, K, N, grid, c = 512, 512, 1024, (2, 2, 2), (1, 0, 1)
    dYg, Wg, Pg = syn.normal_bf16(22, 0, (T, N), 1.0), syn.normal_bf16(22, 1, (K, N), 0.05), syn.normal_bf16(22, 2, (T, K), 1.5)
    p = axo.Problem.make(grid, c, T, K, N)
    _, (M, Kl, Nl, r0, k0, n0) = axo.axo_shard_dims(p)
    dY, W, pre, dX = gu.to_dev(dYg), gu.to_dev(Wg), gu.to_dev(Pg), gu.empty_dev(T, K)
    axo.axo_fc_dgrad_act(p, dY[r0:, n0:].data_ptr(), N, W[k0:, n0:].data_ptr(), N, pre[r0:, k0:].data_ptr(), K,
                         axo.AXO_EPI_BIAS_GELU_TANH, dX[r0:, k0:].data_ptr(), K, None, 0, gu.stream())
    torch.cuda.synchronize()
    ref = oracle.fc_dgrad_act(dYg[r0:r0 + M, n0:n0 + Nl], Wg[k0:k0 + Kl, n0:n0 + Nl], Pg[r0:r0 + M, k0:k0 + Kl],
                              oracle.EPI_BIAS_GELU_TANH)
    out = gu.to_host(dX)
    gu.assert_close(oracle, out[r0:r0 + M, k0:k0 + Kl], ref, "in-place dgrad_act")
    mask = np.ones((T, K), dtype=bool)
    mask[r0:r0 + M, k0:k0 + Kl] = False
    assert (out[mask] == 0x7FC0).all()          # nothing outside the shard was written


@pytest.mark.parametrize("M,Kl,Nl", SHAPES)
def test_wgrad_accumulates_in_fp32(M, Kl, Nl):
    Xb, dYb = syn.normal_bf16(23, 0, (M, Kl), 1.0), syn.normal_bf16(23, 1, (M, Nl), 1.0)
    base = (np.random.default_rng(23).standard_normal((Kl, Nl)) * 30.0).astype(np.float32)
    X, dY = gu.to_dev(Xb), gu.to_dev(dYb)
    dW = torch.from_numpy(base.copy()).to("cuda:0")
    p = P(M, Kl, Nl)
    ref = oracle.fc_wgrad(Xb, dYb)
    scale = np.sqrt(M)                           # typical magnitude of one sum of M products of unit normals
    for rep in (1, 2):                           # accumulate twice: base + product, then + product again
        axo.axo_fc_wgrad_acc(p, X.data_ptr(), Kl, dY.data_ptr(), Nl, dW.data_ptr(), Nl, None, 0, gu.stream())
        torch.cuda.synchronize()
        got = dW.cpu().numpy().astype(np.float64)
        want = base.astype(np.float64) + rep * ref
        # fp32 accumulation of M products plus the fp32 additions into the buffer: a few ulp of the sum's scale
        assert np.max(np.abs(got - want)) <= 2e-5 * (scale + 30.0) * rep, (rep, np.max(np.abs(got - want)))


def test_wgrad_acc_is_unrounded():
    """The product is added without a bf16 rounding: small against large must survive."""
    M, Kl, Nl = 256, 256, 256
    Xb = syn.f32_to_bf16_bits(np.full((M, Kl), 2.0 ** -6, dtype=np.float32))
    dYb = syn.f32_to_bf16_bits(np.full((M, Nl), 2.0 ** -6, dtype=np.float32))
    dW = torch.full((Kl, Nl), 1024.0, dtype=torch.float32, device="cuda:0")
    axo.axo_fc_wgrad_acc(P(M, Kl, Nl), gu.to_dev(Xb).data_ptr(), Kl, gu.to_dev(dYb).data_ptr(), Nl, dW.data_ptr(), Nl,
                         None, 0, gu.stream())
    torch.cuda.synchronize()
    # 256 * 2^-12 = 2^-4 added to 1024: exactly representable in fp32, lost entirely in bf16
    assert torch.all(dW == 1024.0 + 2.0 ** -4)


@pytest.mark.parametrize("M,Nl", [(256, 256), (4096, 1536), (300, 136), (77, 24), (1, 8), (1000, 40), (513, 4104)])
def test_bias_grad(M, Nl):
    dYb = syn.normal_bf16(24, 0, (M, Nl), 1.0)
    dY = gu.to_dev(dYb)
    db = torch.full((Nl,), float("nan"), dtype=torch.float32, device="cuda:0")
    p = P(M, 8, Nl)
    axo.axo_bias_grad(p, dY.data_ptr(), Nl, db.data_ptr(), 0, gu.stream())
    torch.cuda.synchronize()
    ref = oracle.bias_grad(dYb)
    tol = 4e-6 * np.sqrt(M) * 4 + 1e-6           # fp32 sums of M values of unit scale
    got = db.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - ref)) <= tol, np.max(np.abs(got - ref))
    axo.axo_bias_grad(p, dY.data_ptr(), Nl, db.data_ptr(), 1, gu.stream())   # accumulate on top
    torch.cuda.synchronize()
    assert np.max(np.abs(db.cpu().numpy().astype(np.float64) - 2 * ref)) <= 2 * tol
    # run-to-run identical (fixed summation order, no atomics)
    db2 = torch.zeros_like(db)
    axo.axo_bias_grad(p, dY.data_ptr(), Nl, db2.data_ptr(), 0, gu.stream())
    db3 = torch.zeros_like(db)
    axo.axo_bias_grad(p, dY.data_ptr(), Nl, db3.data_ptr(), 0, gu.stream())
    torch.cuda.synchronize()
    assert torch.equal(db2, db3)


@pytest.mark.parametrize("M,Nl", [(256, 256), (4096, 1536), (4096, 6144), (300, 136), (77, 24), (1, 8), (1000, 40),
                                  (513, 4104), (8192, 3584), (100000, 64), (129, 72)])
def test_bias_grad_with_rows_split_over_workgroups(M, Nl):
    """axo_bias_grad_ws against the fp64 oracle: slices of rows per strip, partial sums in the workspace, the
    last workgroup of a strip adds them in slice order.  The workspace is zero-filled once; every call has
    to leave its arrival counters at zero, which the repeated calls on the same workspace rely on."""
    dYb = syn.normal_bf16(26, 0, (M, Nl), 1.0)
    dY = gu.to_dev(dYb)
    p = P(M, 8, Nl)
    nws = axo.axo_bias_grad_workspace_bytes(p)
    ws = torch.zeros(max(nws, 16), dtype=torch.uint8, device="cuda:0")
    wsp = ws.data_ptr() if nws else None
    db = torch.full((Nl,), float("nan"), dtype=torch.float32, device="cuda:0")
    axo.axo_bias_grad_ws(p, dY.data_ptr(), Nl, db.data_ptr(), 0, wsp, nws, gu.stream())
    torch.cuda.synchronize()
    ref = oracle.bias_grad(dYb)
    tol = 4e-6 * np.sqrt(M) * 4 + 1e-6           # fp32 sums of M values of unit scale
    got = db.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - ref)) <= tol, np.max(np.abs(got - ref))
    n_strips = (Nl + 63) // 64
    assert int(ws[:4 * n_strips].view(torch.int32).abs().max()) == 0 if nws else True   # counters back at zero
    axo.axo_bias_grad_ws(p, dY.data_ptr(), Nl, db.data_ptr(), 1, wsp, nws, gu.stream())   # accumulate on top
    torch.cuda.synchronize()
    assert np.max(np.abs(db.cpu().numpy().astype(np.float64) - 2 * ref)) <= 2 * tol
    # run to run identical, whichever workgroup arrives last (fixed summation order, no float atomics)
    # (many back-to-back calls: a slice sum read before it was published would show up here)
    outs = []
    for _ in range(60):
        o = torch.zeros_like(db)
        axo.axo_bias_grad_ws(p, dY.data_ptr(), Nl, o.data_ptr(), 0, wsp, nws, gu.stream())
        outs.append(o)
    torch.cuda.synchronize()
    assert all(torch.equal(outs[0], o) for o in outs[1:])


def test_bias_grad_split_in_place_columns_and_smaller_second_call():
    """A column block addressed inside a wider matrix, then a smaller problem on the same workspace."""
    M, N = 1024, 2048
    dYb = syn.normal_bf16(27, 0, (M, N), 1.0)
    dY = gu.to_dev(dYb)
    p = axo.Problem.make((1, 4, 1), (0, 2, 0), M, 8, N)
    nws = axo.axo_bias_grad_workspace_bytes(p)
    assert nws > 0
    ws = torch.zeros(nws, dtype=torch.uint8, device="cuda:0")
    db = torch.zeros(512, dtype=torch.float32, device="cuda:0")
    axo.axo_bias_grad_ws(p, dY[:, 1024:].data_ptr(), N, db.data_ptr(), 0, ws.data_ptr(), nws, gu.stream())
    p2 = axo.Problem.make((1, 8, 2), (0, 1, 1), M, 8, N)
    nws2 = axo.axo_bias_grad_workspace_bytes(p2)
    assert 0 < nws2 <= nws
    db2 = torch.zeros(256, dtype=torch.float32, device="cuda:0")
    axo.axo_bias_grad_ws(p2, dY[512:, 256:].data_ptr(), N, db2.data_ptr(), 0, ws.data_ptr(), nws, gu.stream())
    torch.cuda.synchronize()
    assert np.max(np.abs(db.cpu().numpy() - oracle.bias_grad(dYb[:, 1024:1536]))) <= 1e-3
    assert np.max(np.abs(db2.cpu().numpy() - oracle.bias_grad(dYb[512:, 256:512]))) <= 1e-3


def test_bias_grad_in_place_columns():
    M, N = 384, 1024
    dYb = syn.normal_bf16(25, 0, (M, N), 1.0)
    dY = gu.to_dev(dYb)
    db = torch.zeros(256, dtype=torch.float32, device="cuda:0")
    axo.axo_bias_grad(axo.Problem.make((1, 4, 1), (0, 2, 0), M, 8, N), dY[:, 512:].data_ptr(), N, db.data_ptr(), 0, gu.stream())
    torch.cuda.synchronize()
    assert np.max(np.abs(db.cpu().numpy() - oracle.bias_grad(dYb[:, 512:768]))) <= 1e-3


def test_layer_step_ext_against_single_calls_and_oracle():
    """axo_layer_step_ext on four layers with buffers of their own: a plain layer, one with all
    three extras (dgrad through the tanh GELU, fp32 weight-gradient accumulation, bias gradient),
    one with the erf GELU and an accumulating bias gradient, and a wide one (4608 columns, a row
    count that is no multiple of the reduction's lane count) whose bias gradient is wide enough to
    ride along in the grouped launch.  The chain is one dependence level, so the fused products
    share a grouped launch with the plain ones.  Every output is checked against the oracle, and
    bit for bit against the single calls."""
    shapes = [(512, 256, 384), (768, 256, 640), (256, 384, 256), (520, 256, 4608)]
    rng = np.random.default_rng(31)
    keep, layers = [], []
    for i, (M, Kl, Nl) in enumerate(shapes):
        Xb, Wb, dYb = (syn.normal_bf16(40 + i, 0, (M, Kl), 1.0), syn.normal_bf16(40 + i, 1, (Kl, Nl), 0.05),
                       syn.normal_bf16(40 + i, 2, (M, Nl), 1.0))
        Pb = syn.normal_bf16(40 + i, 3, (M, Kl), 1.5)
        base32 = (rng.standard_normal((Kl, Nl)) * 30.0).astype(np.float32)
        basedb = (rng.standard_normal(Nl) * 5.0).astype(np.float32)
        t = dict(X=gu.to_dev(Xb), W=gu.to_dev(Wb), dY=gu.to_dev(dYb), pre=gu.to_dev(Pb), Y=gu.empty_dev(M, Nl),
                 dX=gu.empty_dev(M, Kl), dW=gu.empty_dev(Kl, Nl), dW32=torch.from_numpy(base32.copy()).to("cuda:0"),
                 db=torch.from_numpy(basedb.copy()).to("cuda:0"))
        L = axo.Layer(P(M, Kl, Nl), 0, 0, t["X"].data_ptr(), Kl, t["W"].data_ptr(), Nl, None, t["Y"].data_ptr(), Nl,
                      t["dY"].data_ptr(), Nl, t["dX"].data_ptr(), Kl, t["dW"].data_ptr(), Nl)
        if i == 0:
            E = axo.LayerExt.make(L)
        elif i == 1:
            E = axo.LayerExt.make(L, pre=t["pre"].data_ptr(), ldpre=Kl, act_below=axo.AXO_EPI_BIAS_GELU_TANH,
                                  dW32=t["dW32"].data_ptr(), lddw32=Nl, db=t["db"].data_ptr(), accumulate_db=0)
        elif i == 2:
            E = axo.LayerExt.make(L, pre=t["pre"].data_ptr(), ldpre=Kl, act_below=axo.AXO_EPI_BIAS_GELU_ERF,
                                  db=t["db"].data_ptr(), accumulate_db=1)
        else:
            E = axo.LayerExt.make(L, db=t["db"].data_ptr(), accumulate_db=0)
        layers.append(E)
        keep.append((Xb, Wb, dYb, Pb, base32, basedb, t))
    axo.axo_layer_step_ext(layers, None, 0, gu.stream())
    torch.cuda.synchronize()
    for i, ((M, Kl, Nl), (Xb, Wb, dYb, Pb, base32, basedb, t)) in enumerate(zip(shapes, keep)):
        p, tag = P(M, Kl, Nl), f"layer {i}"
        gu.assert_close(oracle, gu.to_host(t["Y"]), oracle.fc_fwd(Xb, Wb), tag + " fwd")
        act = {1: axo.AXO_EPI_BIAS_GELU_TANH, 2: axo.AXO_EPI_BIAS_GELU_ERF}.get(i)
        ref_dx = oracle.fc_dgrad_act(dYb, Wb, Pb, act) if act else oracle.fc_dgrad(dYb, Wb)
        gu.assert_close(oracle, gu.to_host(t["dX"]), ref_dx, tag + " dgrad")
        ref_dw = oracle.fc_wgrad(Xb, dYb)
        if i == 1:   # accumulated in fp32 on top of the initial contents; the bf16 dW was not written
            got = t["dW32"].cpu().numpy().astype(np.float64)
            assert np.max(np.abs(got - (base32.astype(np.float64) + ref_dw))) <= 2e-5 * (np.sqrt(M) + 30.0)
            assert (gu.to_host(t["dW"]) == 0x7FC0).all()
        else:
            gu.assert_close(oracle, gu.to_host(t["dW"]), ref_dw, tag + " wgrad")
            assert np.array_equal(t["dW32"].cpu().numpy(), base32)
        ref_db = oracle.bias_grad(dYb)
        tol = 4e-6 * np.sqrt(M) * 4 + 1e-5
        got_db = t["db"].cpu().numpy().astype(np.float64)
        if i == 0:
            assert np.array_equal(t["db"].cpu().numpy(), basedb)
        elif i in (1, 3):
            assert np.max(np.abs(got_db - ref_db)) <= tol
        else:
            assert np.max(np.abs(got_db - (basedb.astype(np.float64) + ref_db))) <= tol
        if i > 0:    # the stand-alone bias gradient sums in the same order: same bits
            db2 = torch.from_numpy(basedb.copy()).to("cuda:0")
            axo.axo_bias_grad(p, t["dY"].data_ptr(), Nl, db2.data_ptr(), 1 if i == 2 else 0, gu.stream())
            torch.cuda.synchronize()
            assert torch.equal(db2, t["db"])
        # the single calls give the same bits
        Y2, dX2 = gu.empty_dev(M, Nl), gu.empty_dev(M, Kl)
        k = [gu.run_fwd(p, t["X"], t["W"], Y2)]
        if act:
            axo.axo_fc_dgrad_act(p, t["dY"].data_ptr(), Nl, t["W"].data_ptr(), Nl, t["pre"].data_ptr(), Kl, act,
                                 dX2.data_ptr(), Kl, None, 0, gu.stream())
        else:
            k.append(gu.run_dgrad(p, t["dY"], t["W"], dX2))
        torch.cuda.synchronize()
        assert torch.equal(Y2, t["Y"]) and torch.equal(dX2, t["dX"])
        if i == 1:
            dW2 = torch.from_numpy(base32.copy()).to("cuda:0")
            axo.axo_fc_wgrad_acc(p, t["X"].data_ptr(), Kl, t["dY"].data_ptr(), Nl, dW2.data_ptr(), Nl, None, 0, gu.stream())
            torch.cuda.synchronize()
            assert torch.equal(dW2, t["dW32"])
