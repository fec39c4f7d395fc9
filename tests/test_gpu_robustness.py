"""GPU tests of the error paths that need a device to show: degrees given too small (detected by a kernel,
reported as a deferred GP_BAD_ARG; every kernel still stays in bounds and exits normally) and a change of the
triplet-kernel mode between a block's forward and backward call."""
import numpy as np
import pytest
import torch

import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _setup(lib, ctx):
    from dataclasses import replace
    w = replace(synth.get_workload("cfg3", emb=64, emb_rbf=8, cutoff=7.0), max_neighbors=0)
    pos, gptr = synth.box_positions(60, 0.08, 0.9, seed=3)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), w.dims.cutoff, 0)
    W = lib.weights_to_device(synth.weights_G(w.dims, seed=5))
    m, gup = synth.edge_embeddings(e["n_edges"], w.dims.emb, seed=6)
    gb = lib.gp_basis_forward(ctx, w.dims, e, t)
    return w.dims, e, t, W, H.to_dev(m, torch.float32), H.to_dev(gup, torch.float32), gb


def test_understated_degrees_are_reported(lib):
    from paper_2203_09697_amd.binding_g import StackG
    ctx = lib.Context(0)
    lib.gp_set_triplet_mfma(ctx, 1)
    dims, e, t, W, m, gup, gb = _setup(lib, ctx)
    good = StackG(ctx, dims, [W], t, gb)
    ref = good.forward(m).clone()
    lib.gp_deferred_status(ctx)                          # nothing pending
    bad_t = dict(t, max_in_degree=t["max_in_degree"] // 2, max_out_degree=t["max_out_degree"] // 2)
    bad = StackG(ctx, dims, [W], bad_t, gb)
    bad.forward(m)                                       # runs (atoms above the stated degrees are skipped), marks the context
    with pytest.raises(lib.GpError) as err:
        lib.gp_deferred_status(ctx)
    assert err.value.code == -1 and "max_in_degree" in str(err.value)
    lib.gp_deferred_status(ctx)                          # reported once
    bad.forward(m)
    torch.cuda.synchronize()
    with pytest.raises(lib.GpError):                     # ... or by the next block call
        good.forward(m)
    out = good.forward(m)                                # the context is usable afterwards
    lib.gp_deferred_status(ctx)
    assert torch.equal(out, ref)


def test_mode_change_between_forward_and_backward_is_rejected(lib):
    from paper_2203_09697_amd.binding_g import StackG
    ctx = lib.Context(0)
    dims, e, t, W, m, gup, gb = _setup(lib, ctx)
    st = StackG(ctx, dims, [W], t, gb)
    lib.gp_set_triplet_mfma(ctx, 1)                      # forward stores the accumulator as bf16 ...
    st.forward(m)
    lib.gp_set_triplet_mfma(ctx, 0)                      # ... which the vector backward kernels would misread as fp32
    with pytest.raises(lib.GpError) as err:
        st.backward(gup)
    assert err.value.code == -1 and "gp_set_triplet_mfma" in str(err.value)
    lib.gp_set_triplet_mfma(ctx, 1)
    st.forward(m)
    gm, _ = st.backward(gup)
    torch.cuda.synchronize()
    assert np.isfinite(gm.cpu().numpy()).all()
