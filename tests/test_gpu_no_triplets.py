"""GPU parity on a degenerate batch: structures of two atoms (two opposite edges each, and no triplet, since
k -> j -> i needs k != i) plus one isolated atom (no edge at all).  The triplet sum of every block is then
empty: the output comes from the skip paths alone and every weight on the triplet path has a zero gradient.
"""
import numpy as np
import pytest
import torch

import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _pairs(n_pairs, seed):
    rng = np.random.default_rng(seed)
    pos, gptr = [], [0]
    for s in range(n_pairs):
        c = rng.uniform(-1, 1, 3) + 10.0 * s
        u = rng.standard_normal(3)
        pos += [c, c + u / np.linalg.norm(u) * rng.uniform(1.0, 2.5)]
        gptr.append(len(pos))
    pos.append(np.array([500.0, 0.0, 0.0]))
    gptr.append(len(pos))
    return np.array(pos), np.array(gptr)


def _graph(lib, ctx, pos, gptr, cutoff, cap):
    ref = H.oracle_graph(pos, gptr, cutoff, cap)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), cutoff, cap)
    assert len(ref["src"]) == 2 * (len(gptr) - 2) and len(ref["idx_kj"]) == 0
    assert np.array_equal(e["src"].cpu().numpy(), ref["src"]) and t["idx_kj"].numel() == 0
    return ref, e, t


def _check(errs, tol):
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad


def test_block_D_without_triplets(lib, ctx):
    from paper_2203_09697_amd.stack import StackD
    w = synth.get_workload("cfg1")
    dims = w.dims
    pos, gptr = _pairs(7, 0)
    ref, e, t = _graph(lib, ctx, pos, gptr, dims.cutoff, w.max_neighbors)
    E = len(ref["src"])
    W_list = [synth.weights_D(dims, seed=11 + b, bias_scale=0.1) for b in range(2)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=5)
    out_ref, gm_ref, gW_ref = H.oracle_stack_D(ref, H.oracle_basis_D(pos, ref, dims), dims, W_list, m, gup)
    stack = StackD(ctx, dims, [lib.weights_to_device(W) for W in W_list], t, lib.gp_basis_forward(ctx, dims, e, t))
    out = stack.forward(H.to_dev(m, torch.float32))
    gm, gW = stack.backward(H.to_dev(gup, torch.float32))
    torch.cuda.synchronize()
    errs = {"m_out": H.rel_l2(out.cpu().numpy(), out_ref), "grad_m": H.rel_l2(gm.cpu().numpy(), gm_ref)}
    for b in range(2):
        for k in gW_ref[b]:
            errs[f"block{b}.{k}"] = H.rel_l2(gW[b][k].cpu().numpy(), gW_ref[b][k])   # zero reference: absolute norm
    assert np.abs(gW_ref[0]["W_down"]).max() == 0.0 and np.abs(gW_ref[0]["W_ji"]).max() > 0.0
    _check(errs, 1e-4)


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-4), ("bf16", 2e-2)])
def test_block_G_without_triplets(lib, ctx, dtype, tol):
    from paper_2203_09697_amd.binding_g import StackG
    w = synth.get_workload("cfg3", emb=64, int_emb=32, emb_rbf=8, emb_cbf=8, emb_bil=32, num_radial=16,
                           num_spherical=7, cutoff=4.0, dtype=dtype)
    dims = w.dims
    pos, gptr = _pairs(9, 1)
    ref, e, t = _graph(lib, ctx, pos, gptr, dims.cutoff, w.max_neighbors)
    E = len(ref["src"])
    W_list = [synth.weights_G(dims, seed=21)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=6)
    out_ref, gm_ref, gW_ref, grbf_ref = H.oracle_stack_G(ref, H.oracle_basis_G(pos, ref, dims), dims, W_list, m, gup)
    stack = StackG(ctx, dims, [lib.weights_to_device(W) for W in W_list], t, lib.gp_basis_forward(ctx, dims, e, t))
    out = stack.forward(H.to_dev(m, torch.float32))
    grbf = torch.full((E, dims.num_radial), 7.0, dtype=torch.float32, device="cuda:0")
    gm, gW = stack.backward(H.to_dev(gup, torch.float32), grad_rbf=grbf)
    torch.cuda.synchronize()
    errs = {"m_out": H.rel_l2(out.cpu().numpy(), out_ref), "grad_m": H.rel_l2(gm.cpu().numpy(), gm_ref),
            "grad_rbf": H.rel_l2(grbf.cpu().numpy(), grbf_ref)}
    for k in gW_ref[0]:
        errs[k] = H.rel_l2(gW[0][k].cpu().numpy(), gW_ref[0][k])
    assert np.abs(grbf_ref).max() == 0.0
    _check(errs, tol)
