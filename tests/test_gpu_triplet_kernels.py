"""GPU parity of the TripletUpdate + TripletAggr kernels called on their own, in every form the blocks run them,
against the oracle's aggregation functions (oracle.block.triplet_aggregate_D / _G) and automatic differentiation
of the same expressions.  fp32 forms: relative L2 <= 1e-4; forms with bf16 matrix-core operands: <= 2e-2.
The graph is dense enough (in-degrees up to ~90) that the per-centre-atom kernels cut atoms into several shares."""
import numpy as np
import pytest
import torch

import synth
from oracle import basis as obasis
from oracle import block as oblock
from tests import helpers as H

pytestmark = pytest.mark.gpu
F64 = torch.float64


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


@pytest.fixture(scope="module")
def graph(lib, ctx):
    pos, gptr = synth.box_positions(90, 0.08, 0.9, seed=6)
    ref = H.oracle_graph(pos, gptr, 7.0, 0)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), 7.0, 0)
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    ca = obasis.geometry(torch.tensor(pos, dtype=F64), ref["src"], ref["dst"], ref["idx_kj"], ref["idx_ji"])[2]
    order = np.lexsort((ref["idx_ji"], ref["idx_kj"]))                     # kj-major
    deg = np.diff(ref["row_ptr"])
    assert deg.max() > 64
    return dict(ref=ref, t=t, cos=ca, order=order, cos_d=H.to_dev(ca.numpy(), torch.float32),
                cos_kj_d=H.to_dev(ca.numpy()[order], torch.float32))


def _check(pairs, tol):
    errs = {k: (H.rel_l2(a.cpu().numpy(), b), H.row_err(a.cpu().numpy(), b)) for k, (a, b) in pairs.items()}
    print({k: "%.1e / row %.1e" % v for k, v in errs.items()})
    bad = {k: v for k, v in errs.items() if not (v[0] <= tol and v[1] <= (16 if pairs[k][1].ndim == 1 else 4) * tol)}
    assert not bad, bad


@pytest.mark.parametrize("form,F", [(1, 64), (2, 64), (1, 40), (2, 32)], ids=["per-edge", "per-atom", "per-edge odd width", "per-atom 32"])
def test_hadamard_forms(lib, ctx, graph, form, F):
    ref, t = graph["ref"], graph["t"]
    E, T, S, B = len(ref["src"]), len(ref["idx_kj"]), 7, 8
    rng = np.random.default_rng(F + form)
    x = rng.standard_normal((E, F)).astype(np.float32)
    Q = (rng.standard_normal((E, S, B)) * 0.3).astype(np.float32)
    W2 = synth.glorot(rng, (B, F))
    ga = rng.standard_normal((E, F)).astype(np.float32)
    # oracle: s_t = (sum_l Y_l0(t) Q[kj, l, :]) W2;  a = sum_t x[kj] * s_t
    xt, Qt_, W2t = (torch.tensor(v, dtype=F64, requires_grad=True) for v in (x, Q, W2))
    Y = obasis.y_l0(graph["cos"], S)
    kj = torch.as_tensor(ref["idx_kj"], dtype=torch.long)
    p = torch.einsum("tl,tlb->tb", Y, Qt_[kj])
    a_ref = oblock.triplet_aggregate_D(xt, p @ W2t, ref["idx_kj"], ref["idx_ji"], E)
    Bacc_ref = oblock.triplet_aggregate_G(xt, p, ref["idx_kj"], ref["idx_ji"], E)
    gx_ref, gQ_ref, gW2_ref = torch.autograd.grad((a_ref * torch.tensor(ga, dtype=F64)).sum(), [xt, Qt_, W2t])
    Qt_dev = H.to_dev(np.ascontiguousarray(Q.transpose(1, 2, 0).reshape(S * B, E)), torch.float32)
    xd, W2d, gad = H.to_dev(x, torch.float32), H.to_dev(W2, torch.float32), H.to_dev(ga, torch.float32)
    a, Bacc = lib.gp_triplet_hadamard_fwd(ctx, t, form, S, graph["cos_d"], xd, Qt_dev, W2d)
    ws = lib.gp_triplet_workspace(ctx, t, F)
    gx, gQ, gW2 = lib.gp_triplet_hadamard_bwd(ctx, t, form, S, graph["cos_kj_d"], xd, Qt_dev, W2d, gad, ws)
    torch.cuda.synchronize()
    pairs = {"a": (a, a_ref.detach().numpy()), "Bacc": (Bacc, Bacc_ref.detach().numpy()), "grad_x": (gx, gx_ref.numpy()),
             "grad_Q": (gQ, gQ_ref.numpy())}
    if gW2 is not None:
        pairs["grad_W2"] = (gW2, gW2_ref.numpy())
    _check(pairs, 1e-4)


@pytest.mark.parametrize("form,F,C,S,tol", [(1, 64, 16, 7, 1e-4), (2, 64, 16, 7, 2e-2), (3, 64, 16, 7, 2e-2), (2, 128, 16, 7, 2e-2),
                                              (2, 32, 5, 8, 2e-2), (1, 48, 5, 4, 1e-4)],
                         ids=["per-edge", "per-atom", "per-atom two kernels", "per-atom 128", "per-atom narrow", "per-edge odd"])
def test_bilinear_forward_forms(lib, ctx, graph, form, F, C, S, tol):
    ref, t = graph["ref"], graph["t"]
    E = len(ref["src"])
    rng = np.random.default_rng(F + 7 * form + C)
    x = rng.standard_normal((E, F)).astype(np.float32)
    Rad = (rng.standard_normal((E, S, C)) * 0.4).astype(np.float32)
    Y = obasis.y_l0(graph["cos"], S)
    kj = torch.as_tensor(ref["idx_kj"], dtype=torch.long)
    y = torch.einsum("tl,tlc->tc", Y, torch.tensor(Rad, dtype=F64)[kj])
    A_ref = oblock.triplet_aggregate_G(torch.tensor(x, dtype=F64), y, ref["idx_kj"], ref["idx_ji"], E).numpy()
    Radt = H.to_dev(np.ascontiguousarray(Rad.transpose(1, 2, 0).reshape(S * C, E)), torch.float32)
    ws = lib.gp_triplet_workspace(ctx, t, F)
    A = lib.gp_triplet_bilinear_fwd(ctx, t, form, S, C, graph["cos_d"], H.to_dev(x, torch.float32), Radt, ws)
    torch.cuda.synchronize()
    lib.gp_deferred_status(ctx)
    _check({"A": (A.reshape(E * C, F), A_ref.reshape(E * C, F))}, tol)


@pytest.mark.parametrize("form,O,tol,with_ws", [(1, 64, 1e-4, False), (2, 64, 2e-2, True), (2, 64, 2e-2, False), (1, 24, 1e-4, False),
                                                 (2, 128, 2e-2, True), (2, 32, 2e-2, True)],
                         ids=["per-edge", "per-atom", "per-atom whole atom in LDS", "per-edge odd", "per-atom 128", "per-atom 32"])
def test_bilinear_backward_H_and_grad_cos(lib, ctx, graph, form, O, tol, with_ws):
    ref, t, order = graph["ref"], graph["t"], graph["order"]
    E, T, S = len(ref["src"]), len(ref["idx_kj"]), 7
    rng = np.random.default_rng(O + form)
    dz = rng.standard_normal((E, O)).astype(np.float32)
    U = (rng.standard_normal((E, S, O)) * 0.3).astype(np.float32)
    cos = graph["cos"].detach().clone().requires_grad_(True)
    Y = obasis.y_l0(cos, S)
    kj = torch.as_tensor(ref["idx_kj"], dtype=torch.long)
    ji = torch.as_tensor(ref["idx_ji"], dtype=torch.long)
    dzt, Ut = torch.tensor(dz, dtype=F64), torch.tensor(U, dtype=F64)
    # H[e', l, o] = sum_{t: kj(t)=e'} Y_l(t) dz[ji(t), o]
    H_ref = torch.zeros((E, S, O), dtype=F64).index_add(0, kj, Y.detach()[:, :, None] * dzt[ji][:, None, :]).numpy()
    # grad cos_t of  sum_t sum_l Y_l(cos_t) sum_o dz[ji, o] U[kj, l, o]
    L = (Y * torch.einsum("to,tlo->tl", dzt[ji], Ut[kj])).sum()
    (gc_ref,) = torch.autograd.grad(L, cos)
    dzd = H.to_dev(dz, torch.float32)
    ws = lib.gp_triplet_workspace(ctx, t, O) if with_ws else None   # with it the per-atom form is the one-pass kernel
    Hg = lib.gp_triplet_bilinear_bwd_H(ctx, t, form, S, graph["cos_kj_d"], dzd, ws)
    gc = lib.gp_triplet_bilinear_grad_cos(ctx, t, form, S, graph["cos_kj_d"], H.to_dev(U, torch.float32), dzd, ws=ws)
    gc2 = lib.gp_triplet_bilinear_grad_cos(ctx, t, form, S, graph["cos_kj_d"], H.to_dev(U, torch.float32), dzd, grad_cos_kj=gc.clone(),
                                           ws=ws)
    torch.cuda.synchronize()
    lib.gp_deferred_status(ctx)
    _check({"H": (Hg.reshape(E * S, O), H_ref.reshape(E * S, O)), "grad_cos_kj": (gc, gc_ref.numpy()[order]),
            "grad_cos_kj accumulated": (gc2, 2 * gc_ref.numpy()[order])}, tol)


def test_form_errors(lib, ctx, graph):
    t = graph["t"]
    E = t["n_edges"]
    x = torch.zeros((E, 48), dtype=torch.float32, device="cuda:0")
    Radt = torch.zeros((7 * 16, E), dtype=torch.float32, device="cuda:0")
    ws = lib.gp_triplet_workspace(ctx, t, 48)
    with pytest.raises(lib.GpError) as err:
        lib.gp_triplet_bilinear_fwd(ctx, t, lib.TRIPLET_PER_ATOM, 7, 16, graph["cos_d"], x, Radt, ws)    # width 48
    assert err.value.code == -5
    no_lists = {k: v for k, v in t.items() if k not in ("out_list", "out_ptr")}
    with pytest.raises(lib.GpError) as err:
        lib.gp_triplet_bilinear_fwd(ctx, no_lists, lib.TRIPLET_PER_ATOM, 7, 16, graph["cos_d"], x, Radt, ws)
    assert err.value.code == -1
    with pytest.raises(lib.GpError) as err:
        lib.gp_triplet_bilinear_fwd(ctx, t, 9, 7, 16, graph["cos_d"], x, Radt, ws)
    assert err.value.code == -1
