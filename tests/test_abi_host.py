"""Host-side tests of the C ABI (no GPU): the library loads, exports every function that
include/axo.h declares, derives shards the way Section 3.2 of the paper cuts I and W over the
grid, and turns every malformed argument into its status code before any HIP call."""
import ctypes
import glob
import os
import re

import pytest

import oracle
import paper_2305_13525_amd as axo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "axo.h")

OK, BAD_GRID, BAD_COORD, INDIVISIBLE, NULL_PTR, MISALIGNED, BAD_LD, WORKSPACE, BAD_EPI, HIP, BAD_SIZE, BAD_ARG, NO_MEMORY, TOO_LARGE = (
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10, -11, -12, -13)


def declared_functions():
    names = set()
    for header in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(axo_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"axo_fc_fwd", "axo_fc_dgrad", "axo_fc_wgrad", "axo_layer_step", "axo_shard_dims",
            "axo_workspace_bytes", "axo_status_string", "axo_version",
            "axo_layer_step_workspace_bytes", "axo_layer_step_ordered", "axo_layer_step_levels", "axo_layer_step_ext",
            "axo_comm_rank_configs",
            "axo_comm_layer_time"} <= set(names)
    lib = ctypes.CDLL(axo.library_path())
    for n in names:
        assert hasattr(lib, n), n
    assert axo.axo_version() == 1


def test_struct_layout_matches_header():
    assert ctypes.sizeof(axo.Problem) == 56
    assert axo.Problem.T.offset == 24 and axo.Problem.transposed.offset == 48
    assert ctypes.sizeof(axo.Layer) == 56 + 8 + 13 * 8
    assert axo.Layer.X.offset == 64 and axo.Layer.bias.offset == 96 and axo.Layer.dW.offset == 152
    assert ctypes.sizeof(axo.LayerExt) == ctypes.sizeof(axo.Layer) + 5 * 8 + 8
    assert axo.LayerExt.pre.offset == 168 and axo.LayerExt.db.offset == 200 and axo.LayerExt.act_below.offset == 208


def test_status_strings():
    seen = set()
    for s in range(0, -14, -1):
        t = axo.axo_status_string(s)
        assert t and t != "unknown status" and t not in seen
        seen.add(t)
    assert axo.axo_status_string(-99) == "unknown status"


@pytest.mark.parametrize("transposed", [0, 1])
def test_shard_dims_match_oracle_slices(transposed):
    T, K, N, grid = 48, 72, 120, (2, 3, 4)
    for ix in range(2):
        for iy in range(3):
            for iz in range(4):
                p = axo.Problem.make(grid, (ix, iy, iz), T, K, N, transposed)
                rc, (M, Kl, Nl, row0, k0, n0) = axo.axo_shard_dims(p)
                rt, rk, rn = oracle.shard_slices(T, K, N, grid, (ix, iy, iz), bool(transposed))
                assert (row0, row0 + M) == (rt.start, rt.stop)
                assert (k0, k0 + Kl) == (rk.start, rk.stop)
                assert (n0, n0 + Nl) == (rn.start, rn.stop)


def test_benchmark_shard_shapes():
    want = {((2, 2, 4), 16384, 4096, 12288): (4096, 2048, 6144),
            ((4, 2, 8), 32768, 8192, 32768): (4096, 2048, 16384),
            ((2, 4, 8), 32768, 32768, 8192): (4096, 16384, 2048),
            ((8, 8, 4), 16384, 12288, 36864): (4096, 1536, 4608),
            ((8, 8, 4), 16384, 49152, 12288): (4096, 6144, 1536)}
    for (grid, T, K, N), shard in want.items():
        rc, d = axo.axo_shard_dims(axo.Problem.make(grid, (0, 0, 0), T, K, N))
        assert d[:3] == shard


def test_shard_dims_errors():
    mk = axo.Problem.make
    sd = lambda p: axo.axo_shard_dims(p, check=False)[0]
    assert sd(None) == NULL_PTR
    assert sd(mk((0, 1, 1), (0, 0, 0), 8, 8, 8)) == BAD_GRID
    assert sd(mk((1, -2, 1), (0, 0, 0), 8, 8, 8)) == BAD_GRID
    assert sd(mk((2, 2, 2), (2, 0, 0), 8, 8, 8)) == BAD_COORD
    assert sd(mk((2, 2, 2), (0, 0, -1), 8, 8, 8)) == BAD_COORD
    assert sd(mk((2, 2, 2), (0, 0, 0), 9, 8, 8)) == INDIVISIBLE
    assert sd(mk((2, 2, 2), (0, 0, 0), 8, 9, 8)) == INDIVISIBLE
    assert sd(mk((2, 4, 2), (0, 0, 0), 8, 8, 10)) == INDIVISIBLE
    assert sd(mk((2, 4, 2), (0, 0, 0), 8, 10, 8, 1)) == INDIVISIBLE   # transposed: K over Gy
    assert sd(mk((2, 4, 2), (0, 0, 0), 8, 8, 10, 1)) == OK            # transposed: N over Gx
    assert sd(mk((1, 1, 1), (0, 0, 0), -1, 8, 8)) == BAD_SIZE
    assert sd(mk((1, 1, 1), (0, 0, 0), 2 ** 33, 8, 8)) == BAD_SIZE
    assert sd(mk((1, 1, 1), (0, 0, 0), 8, 8, 8, 2)) == BAD_ARG
    bad = mk((1, 1, 1), (0, 0, 0), 8, 8, 8)
    bad.reserved = 7
    assert sd(bad) == BAD_ARG
    with pytest.raises(axo.AxoError):
        axo.axo_shard_dims(mk((0, 1, 1), (0, 0, 0), 8, 8, 8))


# The pointer checks below never reach a HIP call: every call is malformed on purpose, so the
# fake addresses are never dereferenced.
A = 0x10000  # 16-byte aligned fake device address
A1, A2, A3, A4, A5, A6, A7 = (A + i * 0x100000 for i in range(1, 8))  # further ones, far enough apart for any matrix here


def test_fwd_argument_errors():
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48)
    f = lambda **kw: axo.axo_fc_fwd(**{**dict(p=p, X=A, ldx=32, W=A, ldw=48, bias=None, epilogue=0, Y=A, ldy=48,
                                            check=False), **kw})
    assert f(p=None) == NULL_PTR
    assert f(X=None) == NULL_PTR and f(W=None) == NULL_PTR and f(Y=None) == NULL_PTR
    assert f(ldx=24) == BAD_LD and f(ldw=40) == BAD_LD and f(ldy=8) == BAD_LD
    assert f(ldx=36) == MISALIGNED and f(X=A + 2) == MISALIGNED and f(Y=A + 8) == MISALIGNED
    assert f(epilogue=4) == BAD_EPI and f(epilogue=-1) == BAD_EPI
    assert f(epilogue=1, bias=None) == BAD_EPI
    assert f(epilogue=2, bias=A + 2) == MISALIGNED
    assert f(p=axo.Problem.make((2, 1, 1), (0, 0, 0), 64, 33, 48)) == INDIVISIBLE


def test_dgrad_wgrad_argument_errors():
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48)
    d = lambda **kw: axo.axo_fc_dgrad(**{**dict(p=p, dY=A, lddy=48, W=A, ldw=48, dX=A, lddx=32, check=False), **kw})
    w = lambda **kw: axo.axo_fc_wgrad(**{**dict(p=p, X=A, ldx=32, dY=A, lddy=48, dW=A, lddw=48, check=False), **kw})
    assert d(dY=None) == NULL_PTR and d(W=None) == NULL_PTR and d(dX=None) == NULL_PTR
    assert d(lddy=40) == BAD_LD and d(lddx=24) == BAD_LD and d(ldw=50) == MISALIGNED
    assert w(X=None) == NULL_PTR and w(dY=None) == NULL_PTR and w(dW=None) == NULL_PTR
    assert w(ldx=16) == BAD_LD and w(lddw=40) == BAD_LD and w(dW=A + 4) == MISALIGNED
    assert d(p=None) == NULL_PTR and w(p=None) == NULL_PTR


def test_output_must_not_share_bytes_with_an_input():
    """The header's rule, enforced on the host: the kernels write output tiles while other workgroups
    still read the operands (and compute the overlap of a ragged output's tiles twice), so a product
    written over one of its own inputs is refused.  Sharing a buffer without sharing bytes is fine."""
    M, K, N = 64, 32, 48
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), M, K, N)
    fwd = lambda X, ldx, Y, ldy: axo.axo_fc_fwd(p, X, ldx, A1, N, None, 0, Y, ldy, check=False)
    # the route query plans a product without launching it; here the planners' verdict is all we want,
    # so every call below is made on a problem with nothing to launch where it would pass
    none = axo.Problem.make((1, 1, 1), (0, 0, 0), M, K, 0)
    assert axo.axo_fc_fwd(none, A, K, A1, 8, None, 0, A, 8, check=False) == OK      # no output element: no overlap
    assert fwd(A, K, A, N) == BAD_ARG                                               # Y over X
    assert fwd(A, K, A + (M - 1) * K * 2 + K * 2 - 16, N) == BAD_ARG                # Y begins on X's last 16 bytes
    assert axo.axo_fc_dgrad(p, A, N, A1, N, A1 + 64, K, check=False) == BAD_ARG      # dX inside W
    assert axo.axo_fc_wgrad(p, A, K, A1, N, A1, N, check=False) == BAD_ARG           # dW over dY
    # X and Y as interleaved column blocks of one buffer with rows of K + N elements share no byte:
    # that call passes validation (and would go on to launch, so it is asked as a route here)
    levels = axo.axo_layer_step_levels(
        [axo.Layer(p, 0, 0, A, K + N, A1, N, None, A + K * 2, K + N, A3, N, A4, K, A5, N)], check=False)
    assert levels[0] == OK
    # ... while shifting Y one 16-byte step to the left runs it into X's columns
    levels = axo.axo_layer_step_levels(
        [axo.Layer(p, 0, 0, A, K + N, A1, N, None, A + K * 2 - 16, K + N, A3, N, A4, K, A5, N)], check=False)
    assert levels[0] == BAD_ARG


def test_routes_follow_shape_and_leading_dimensions():
    """axo_fc_route: which kernels a product takes is decided on the host from the shard shape and the
    leading dimensions.  The tuned kernel forms 32-bit byte offsets inside an operand tile, so the span
    it walks must stay below 4 GiB; for wgrad that span is the token count ROUNDED UP to 128."""
    mk = lambda M, K, N: axo.Problem.make((1, 1, 1), (0, 0, 0), M, K, N)
    route = lambda p, op, a, b, c: axo.axo_fc_route(p, op, a, b, c)[1]
    FWD, DG, WG = axo.AXO_OP_FWD, axo.AXO_OP_DGRAD, axo.AXO_OP_WGRAD
    p = mk(4096, 2048, 6144)                                    # benchmark config 2: all three tiled
    assert [route(p, FWD, 2048, 6144, 6144), route(p, DG, 6144, 6144, 2048), route(p, WG, 2048, 6144, 6144)] == [1, 1, 1]
    assert route(mk(0, 32, 48), FWD, 32, 48, 48) == axo.AXO_ROUTE_NONE
    assert route(mk(77, 40, 24), FWD, 40, 24, 24) == axo.AXO_ROUTE_GENERAL
    assert route(mk(520, 384, 264), FWD, 384, 264, 264) == axo.AXO_ROUTE_COVERED
    assert route(mk(520, 264, 384), WG, 264, 384, 384) == axo.AXO_ROUTE_COVERED
    assert route(mk(1000, 256, 384), WG, 256, 384, 384) == axo.AXO_ROUTE_TILED       # any token count
    # 450 tokens, 4.3 M elements apart: 450 rows span 3.87 GB, the 512 walked rows 4.4 GB
    assert route(mk(450, 256, 384), WG, 4_300_000, 4_300_000, 384) == axo.AXO_ROUTE_GENERAL
    assert route(mk(384, 256, 384), WG, 4_300_000, 4_300_000, 384) == axo.AXO_ROUTE_TILED    # 384 = 3 * 128 rows: 3.3 GB
    # 131005 tokens 16392 elements apart: the valid rows end just below the limit, row 131071 does not
    assert (131005 * 16392 + 256) * 2 < 0xFFFF0000 < (131072 * 16392 + 256) * 2
    assert route(mk(131005, 256, 384), WG, 16392, 16392, 384) == axo.AXO_ROUTE_GENERAL
    assert route(mk(130944, 256, 384), WG, 16392, 16392, 384) == axo.AXO_ROUTE_TILED
    # errors are those of the product's own argument checks
    assert axo.axo_fc_route(mk(64, 32, 48), FWD, 24, 48, 48, check=False)[0] == BAD_LD
    assert axo.axo_fc_route(mk(64, 32, 48), 5, 32, 48, 48, check=False)[0] == BAD_ARG
    assert axo.library().axo_fc_route(None, 0, 8, 8, 8, None) == NULL_PTR


def test_workspace_query():
    """No product needs device workspace at present; the query is total and never fails."""
    mk = axo.Problem.make
    for op in (axo.AXO_OP_FWD, axo.AXO_OP_DGRAD, axo.AXO_OP_WGRAD):
        assert axo.axo_workspace_bytes(mk((2, 2, 4), (0, 0, 0), 16384, 4096, 12288), op) == 0
        assert axo.axo_workspace_bytes(mk((1, 1, 1), (0, 0, 0), 1000, 520, 264), op) == 0
    assert axo.axo_workspace_bytes(mk((0, 1, 1), (0, 0, 0), 8, 8, 8), axo.AXO_OP_FWD) == 0   # invalid problem
    assert axo.axo_workspace_bytes(mk((1, 1, 1), (0, 0, 0), 8, 8, 8), 7) == 0                # unknown op


def test_empty_shards_need_no_device():
    # M == 0 or Nl == 0: valid, nothing is launched, so this runs without a GPU
    p0 = axo.Problem.make((1, 1, 1), (0, 0, 0), 0, 32, 48)
    assert axo.axo_fc_fwd(p0, A, 32, A, 48, None, 0, A, 48, check=False) == OK
    assert axo.axo_fc_dgrad(p0, A, 48, A, 48, A, 32, check=False) == OK
    pn = axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 0)
    assert axo.axo_fc_fwd(pn, A, 32, A, 8, None, 0, A, 8, check=False) == OK
    assert axo.axo_fc_wgrad(pn, A, 32, A, 8, A, 8, check=False) == OK


@pytest.mark.parametrize("entry", ["axo_layer_step", "axo_layer_step_ordered"])
def test_layer_step_validates_whole_chain_first(entry):
    step = getattr(axo, entry)
    # T == 0 and N == 0: none of the three products has an output element, so nothing launches
    good = axo.Layer(axo.Problem.make((1, 1, 1), (0, 0, 0), 0, 32, 0), 0, 0, A, 32, A, 8, None, A, 8, A, 8,
                     A, 32, A, 8)
    bad = axo.Layer(axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48), 0, 0, A, 32, A1, 48, None, A2, 48, A3, 48,
                    None, 32, A5, 48)  # dX missing
    assert step([], check=False) == OK
    assert step([good], check=False) == OK  # empty shard: no launch
    assert step([good, bad], check=False) == NULL_PTR
    worse = axo.Layer(axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48), 9, 0, A, 32, A, 48, None, A, 48, A, 48,
                      A, 32, A, 48)
    assert step([worse], check=False) == BAD_EPI
    # an output that shares bytes with an input of its own product is refused (here dX over dY)
    alias = axo.Layer(axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48), 0, 0, A, 32, A1, 48, None, A2, 48, A3, 48,
                      A3, 32, A5, 48)
    assert step([good, alias], check=False) == BAD_ARG
    assert getattr(axo.library(), entry)(None, 2, None, 0, None) == NULL_PTR
    assert getattr(axo.library(), entry)(None, -1, None, 0, None) == BAD_ARG
    assert axo.axo_layer_step_workspace_bytes([good, bad]) >= 0


def test_dependence_levels_are_decided_on_byte_ranges():
    """axo_layer_step_levels (host only; the addresses are made up and never dereferenced): the
    dependence analysis by which axo_layer_step decides which products may share a launch.
    Product order: fwd of layers 0..n-1, then dgrad, wgrad of layers n-1..0."""
    M, K, N = 64, 32, 48
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), M, K, N)
    base = 1 << 20

    def layer(X, W, Y, dY, dX, dW, ldx=K, ldy=N):
        return axo.Layer(p, 0, 0, X, ldx, W, N, None, Y, ldy, dY, N, dX, K, dW, N)

    def levels(ls):
        rc, n, lv = axo.axo_layer_step_levels(ls)
        assert rc == OK and (n == (max(lv) + 1 if lv else 0))
        return lv

    step = 1 << 16  # far more than any of the matrices spans
    a = [base + i * step for i in range(16)]
    l0 = layer(a[0], a[1], a[2], a[3], a[4], a[5])
    l1 = layer(a[6], a[7], a[8], a[9], a[10], a[11])
    assert axo.axo_layer_step_levels([]) == (OK, 0, [])
    assert levels([l0]) == [0, 0, 0]
    # layers with buffers of their own: one level         fwd0 fwd1 dg1 wg1 dg0 wg0
    assert levels([l0, l1]) == [0, 0, 0, 0, 0, 0]
    # the same weight read by two layers is no dependence
    assert levels([l0, layer(a[6], a[1], a[8], a[9], a[10], a[11])]) == [0] * 6
    # layer one reads what layer zero writes: its fwd and its wgrad (which reads X) wait for fwd 0
    assert levels([l0, layer(a[2], a[7], a[8], a[9], a[10], a[11])]) == [0, 1, 0, 1, 0, 0]
    # layer zero's dY is layer one's dX: layer zero's backward pair waits for dgrad 1
    assert levels([l0, layer(a[6], a[7], a[8], a[9], a[3], a[11])]) == [0, 0, 0, 0, 1, 1]
    # both at once, the layout of a real two-layer step
    assert levels([l0, layer(a[2], a[7], a[8], a[9], a[3], a[11])]) == [0, 1, 0, 1, 1, 1]
    # two layers write the same dW: the later write (wgrad 0) waits for the earlier (wgrad 1)
    assert levels([l0, layer(a[6], a[7], a[8], a[9], a[10], a[5])]) == [0, 0, 0, 0, 0, 1]
    # write after read: layer one's Y is the buffer layer zero's forward reads as X; fwd 1 waits for
    # fwd 0, and wgrad 0, which in program order reads that buffer after fwd 1 has rewritten it, for fwd 1
    assert levels([l0, layer(a[6], a[7], a[0], a[9], a[10], a[11])]) == [0, 1, 0, 0, 0, 2]
    # an output that begins on the last 16 bytes of one of its own inputs is refused; one that
    # begins right behind it is fine.  X spans (M - 1) * K + K elements
    x_bytes = ((M - 1) * K + K) * 2
    assert axo.axo_layer_step_levels([layer(a[0], a[1], a[0] + x_bytes - 16, a[3], a[4], a[5])], check=False)[0] == BAD_ARG
    assert levels([layer(a[0], a[1], a[0] + x_bytes, a[3], a[4], a[5])]) == [0, 0, 0]
    # the same 16 bytes shared with an input of ANOTHER product are a dependence, not an error:
    # layer one's Y ends on the first bytes of layer zero's X, which wgrad 0 reads afterwards
    assert levels([l0, layer(a[6], a[7], a[0] - ((M - 1) * N + N) * 2 + 16, a[9], a[10], a[11])]) == [0, 1, 0, 0, 0, 2]
    # column blocks interleaved in one buffer (ld twice the row length) count as overlapping
    assert levels([layer(a[0], a[1], a[2], a[3], a[4], a[5], ldy=2 * N),
                   layer(a[6], a[7], a[2] + 2 * N, a[9], a[10], a[11], ldy=2 * N)]) == [0, 1, 0, 0, 0, 0]
    # a chain of three: each forward waits for the one before
    l2 = layer(a[8], a[12], a[13], a[14], a[15], base + 16 * step)
    assert levels([l0, layer(a[2], a[7], a[8], a[9], a[10], a[11]), l2])[:3] == [0, 1, 2]
    # 256 layers (768 products) are still analysed, one more and the chain keeps its order
    many = [layer(*[base + (7 * i + k) * step for k in range(6)]) for i in range(257)]
    assert axo.axo_layer_step_levels(many[:256])[1] == 1
    rc, n, lv = axo.axo_layer_step_levels(many)
    assert (rc, n) == (OK, 771) and lv == list(range(771))
    # validation comes first
    bad = axo.Layer(p, 0, 0, a[0], K, a[1], N, None, a[2], N, a[3], N, None, K, a[5], N)
    assert axo.axo_layer_step_levels([bad], check=False)[0] == NULL_PTR
    assert axo.library().axo_layer_step_levels(None, 0, None, None) == NULL_PTR


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2305_13525_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libaxo.so")
    with pytest.raises(FileNotFoundError):
        b.library()


def test_backward_extras_argument_errors():
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48)
    # dgrad through an activation: act must name one of the two GELUs; pre is a [M x Kl] matrix
    assert axo.axo_fc_dgrad_act(p, A, 48, A1, 48, A2, 32, 1, A3, 32, check=False) == BAD_EPI
    assert axo.axo_fc_dgrad_act(p, A, 48, A1, 48, None, 32, 2, A3, 32, check=False) == NULL_PTR
    assert axo.axo_fc_dgrad_act(p, A, 48, A1, 48, A2, 24, 3, A3, 32, check=False) == BAD_LD
    assert axo.axo_fc_dgrad_act(p, A, 40, A1, 48, A2, 32, 2, A3, 32, check=False) == BAD_LD
    assert axo.axo_fc_dgrad_act(p, A, 48, A1, 48, A2, 32, 2, A2, 32, check=False) == BAD_ARG   # dX over pre
    # fp32 accumulation: ld in floats, multiple of 4, 16-byte aligned base
    assert axo.axo_fc_wgrad_acc(p, A, 32, A1, 48, None, 48, check=False) == NULL_PTR
    assert axo.axo_fc_wgrad_acc(p, A, 32, A1, 48, A2, 40, check=False) == BAD_LD
    assert axo.axo_fc_wgrad_acc(p, A, 32, A1, 48, A2, 50, check=False) == MISALIGNED
    assert axo.axo_fc_wgrad_acc(p, A, 32, A1, 48, A2 + 8, 48, check=False) == MISALIGNED
    assert axo.axo_fc_wgrad_acc(p, A, 24, A1, 48, A2, 48, check=False) == BAD_LD
    # the fp32 matrix is twice as large in bytes as the bf16 stand-in: its tail reaching into X is caught
    assert axo.axo_fc_wgrad_acc(p, A, 32, A1, 48, A - 32 * 48 * 4 + 16, 48, check=False) == BAD_ARG
    # bias gradient
    assert axo.axo_bias_grad(p, A, 48, None, 0, check=False) == NULL_PTR
    assert axo.axo_bias_grad(p, A, 48, A1 + 2, 0, check=False) == MISALIGNED
    assert axo.axo_bias_grad(p, A, 48, A1, 2, check=False) == BAD_ARG
    assert axo.axo_bias_grad(p, A, 40, A1, 0, check=False) == BAD_LD
    assert axo.axo_bias_grad(p, A, 48, A + 96, 0, check=False) == BAD_ARG                      # db inside dY
    # nothing to do: valid without a device
    pn = axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 0)
    assert axo.axo_bias_grad(pn, A, 8, A, 0, check=False) == OK
    assert axo.axo_fc_wgrad_acc(pn, A, 32, A, 8, A, 8, check=False) == OK
    p0 = axo.Problem.make((1, 1, 1), (0, 0, 0), 0, 32, 48)
    assert axo.axo_fc_dgrad_act(p0, A, 48, A, 48, A, 32, 2, A, 32, check=False) == OK


def test_bias_grad_workspace_query_and_errors():
    mk = lambda M, N: axo.Problem.make((1, 1, 1), (0, 0, 0), M, 8, N)
    # 96 strips of 64 columns, 4 slices of 1024 rows (384 workgroups):
    # 512 bytes of counters (96 * 4 rounded up to 256) + 4 * 6144 floats
    assert axo.axo_bias_grad_workspace_bytes(mk(4096, 6144)) == 512 + 4 * 6144 * 4
    assert axo.axo_bias_grad_workspace_bytes(mk(4096, 16384)) == 1024 + 2 * 16384 * 4
    assert axo.axo_bias_grad_workspace_bytes(mk(77, 24)) == 0            # too few rows to split
    assert axo.axo_bias_grad_workspace_bytes(mk(255, 24)) == 0
    assert axo.axo_bias_grad_workspace_bytes(mk(256, 24)) == 256 + 2 * 24 * 4
    assert axo.axo_bias_grad_workspace_bytes(axo.Problem.make((0, 1, 1), (0, 0, 0), 8, 8, 8)) == 0   # invalid problem
    p = mk(4096, 6144)
    need = axo.axo_bias_grad_workspace_bytes(p)
    B1, B2 = 1 << 40, 2 << 40                                             # far beyond dY's 50 MB
    f = lambda **kw: axo.axo_bias_grad_ws(**{**dict(p=p, dY=A, lddy=6144, db=B1, accumulate=0, ws=B2, ws_bytes=need,
                                                    check=False), **kw})
    assert f(ws=None) == WORKSPACE and f(ws_bytes=need - 1) == WORKSPACE and f(ws=B2 + 8) == MISALIGNED
    assert f(db=None) == NULL_PTR and f(lddy=6136) == BAD_LD and f(accumulate=3) == BAD_ARG
    assert f(db=A + 128) == BAD_ARG                                       # db inside dY
    # nothing to do: valid without a device or a workspace
    assert axo.axo_bias_grad_ws(mk(64, 0), A, 8, A1, 0, None, 0, check=False) == OK


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's share; asked for more it has to say so and exit non-zero
    (decided before anything touches a GPU, so this runs anywhere)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "--gpus must be 1" in (r.stdout + r.stderr)


def test_layer_step_ext_validation():
    """The extras of axo_layer_step_ext are validated like the single calls, before any launch."""
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), 64, 32, 48)
    base = axo.Layer(p, 0, 0, A, 32, A1, 48, None, A2, 48, A3, 48, A4, 32, A5, 48)
    ext = axo.LayerExt.make
    step = lambda ls: axo.axo_layer_step_ext(ls, check=False)
    assert step([]) == OK
    assert step([ext(base, act_below=2)]) == BAD_EPI                        # an activation without its pre-activation
    assert step([ext(base, pre=A6, ldpre=32, act_below=0)]) == BAD_EPI      # a pre-activation without an activation
    assert step([ext(base, pre=A6, ldpre=32, act_below=1)]) == BAD_EPI      # bias alone is no activation
    assert step([ext(base, pre=A6, ldpre=24, act_below=2)]) == BAD_LD
    assert step([ext(base, pre=A4, ldpre=32, act_below=2)]) == BAD_ARG      # dX written over the pre-activation it reads
    assert step([ext(base, dW32=A7, lddw32=40)]) == BAD_LD
    assert step([ext(base, dW32=A7, lddw32=50)]) == MISALIGNED
    assert step([ext(base, dW32=A3, lddw32=48)]) == BAD_ARG                 # the fp32 gradient over dY
    assert step([ext(base, db=A7 + 2)]) == MISALIGNED
    assert step([ext(base, db=A7, accumulate_db=2)]) == BAD_ARG
    assert step([ext(base, db=A3 + 64)]) == BAD_ARG                         # the bias gradient inside dY
    no_dw = axo.Layer(p, 0, 0, A, 32, A1, 48, None, A2, 48, A3, 48, A4, 32, None, 48)
    assert step([ext(no_dw)]) == NULL_PTR                                    # plain wgrad needs layer.dW ...
    empty = axo.Problem.make((1, 1, 1), (0, 0, 0), 0, 32, 0)                # (nothing to launch: valid anywhere)
    nothing = axo.Layer(empty, 0, 0, A, 32, A, 8, None, A, 8, A, 8, A, 32, None, 8)
    assert step([ext(nothing, dW32=A, lddw32=8)]) == OK                      # ... the fp32 one does not
    assert axo.library().axo_layer_step_ext(None, 1, None, 0, None) == NULL_PTR
    assert axo.library().axo_layer_step_ext(None, -1, None, 0, None) == BAD_ARG


def test_dependence_levels_on_random_chains():
    """Property check of axo_layer_step_levels on seeded random chains whose buffers are drawn from
    a small pool (so that reads and writes collide often).  The byte ranges and the conflict rule
    are restated here in Python; the library's levels must (i) put every product above all earlier
    products it conflicts with and (ii) be minimal: each product sits exactly one above the
    highest conflicting earlier product, or at 0."""
    import random
    M, K, N = 64, 32, 48
    p = axo.Problem.make((1, 1, 1), (0, 0, 0), M, K, N)
    base, slot = 1 << 22, 1 << 15            # slots are larger than any matrix here (at most 64 * 48 * 2 bytes)
    span = lambda rows, cols, ld: ((rows - 1) * ld + cols) * 2

    def products(lay):
        X, W, Y, dY, dX, dW = lay
        rng = lambda ptr, rows, cols, ld: (ptr, ptr + span(rows, cols, ld))
        fwd = ([rng(X, M, K, K), rng(W, K, N, N)], rng(Y, M, N, N))
        dg = ([rng(dY, M, N, N), rng(W, K, N, N)], rng(dX, M, K, K))
        wg = ([rng(X, M, K, K), rng(dY, M, N, N)], rng(dW, K, N, N))
        return fwd, dg, wg

    def conflict(a, b):      # a earlier than b
        ov = lambda r, q: r[0] < q[1] and q[0] < r[1]
        return ov(a[1], b[1]) or any(ov(a[1], r) for r in b[0]) or any(ov(r, b[1]) for r in a[0])

    rnd = random.Random(7)
    for case in range(150):
        n = rnd.randint(1, 6)
        pool = [base + i * slot for i in range(rnd.randint(6, 6 * n + 2))]
        # half-slot offsets make partial overlaps as well as exact aliases
        pick = lambda: rnd.choice(pool) + rnd.choice((0, 0, 0, 1 << 11))
        lays = []
        ov = lambda r, q: r[0] < q[1] and q[0] < r[1]
        while len(lays) < n:
            lay = tuple(pick() for _ in range(6))
            # an output that shares bytes with an input of its own product is refused by the library
            # (all matrices here are contiguous, so sharing bytes is the same as overlapping ranges)
            if any(ov(out, r) for ins, out in products(lay) for r in ins):
                continue
            lays.append(lay)
        layers = [axo.Layer(p, 0, 0, X, K, W, N, None, Y, N, dY, N, dX, K, dW, N) for X, W, Y, dY, dX, dW in lays]
        rc, n_levels, lv = axo.axo_layer_step_levels(layers)
        assert rc == OK and len(lv) == 3 * n
        prods = [products(l)[0] for l in lays]                       # program order: forwards ...
        for l in reversed(lays):                                      # ... then dgrad, wgrad of layers n-1..0
            prods += list(products(l)[1:])
        for j in range(3 * n):
            want = 0
            for i in range(j):
                if conflict(prods[i], prods[j]):
                    want = max(want, lv[i] + 1)
            assert lv[j] == want, (case, j, lv)
        assert n_levels == max(lv) + 1
