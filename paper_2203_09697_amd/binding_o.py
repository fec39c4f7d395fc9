"""ctypes binding of the output block (gp_output_*) and a variant-D model with one output block
after every interaction block.  Argument marshalling, allocation and call sequencing only."""
import ctypes as C

import torch

from . import binding as B

__all__ = ["gp_output_workspace", "gp_output_forward", "gp_output_backward", "ModelD"]

GP_MAX_OUT_LAYERS = 4


class _WeightsOut(C.Structure):
    _fields_ = [("W_rbf", C.c_void_p), ("W_up", C.c_void_p), ("W", C.c_void_p * GP_MAX_OUT_LAYERS),
                ("b", C.c_void_p * GP_MAX_OUT_LAYERS), ("w_final", C.c_void_p)]


def n_layers_of(w):
    k = 0
    while f"W{k}" in w:
        k += 1
    return k


def _out(w):
    s = _WeightsOut(W_rbf=B._ptr(w["W_rbf"]), W_up=B._ptr(w["W_up"]), w_final=B._ptr(w["w_final"]))
    for k in range(n_layers_of(w)):
        s.W[k] = B._ptr(w[f"W{k}"])
        s.b[k] = B._ptr(w[f"b{k}"])
    return s


def _shape(w):
    R, emb = w["W_rbf"].shape
    return emb, w["W_up"].shape[1], R, n_layers_of(w)


def gp_output_workspace(emb, out_emb, num_radial, n_layers, n_atoms, n_edges):
    a, b = C.c_size_t(), C.c_size_t()
    rc = B.load().gp_output_workspace(C.c_int32(emb), C.c_int32(out_emb), C.c_int32(num_radial), C.c_int32(n_layers),
                                      C.c_int64(n_atoms), C.c_int64(n_edges), C.byref(a), C.byref(b))
    if rc != 0:
        raise B.GpError(rc, "gp_output_workspace")
    return a.value, b.value


def gp_output_forward(ctx, w, m, rbf, row_ptr, graph_ptr, accumulate, energy, saved, scratch):
    emb, out_emb, R, L = _shape(w)
    ws = _out(w)
    ctx.check(B.load().gp_output_forward(
        ctx._h, C.c_int32(emb), C.c_int32(out_emb), C.c_int32(R), C.c_int32(L), C.byref(ws), B._ptr(m), B._ptr(rbf),
        B._ptr(row_ptr), B._ptr(graph_ptr), C.c_int64(row_ptr.shape[0] - 1), C.c_int64(m.shape[0]),
        C.c_int32(graph_ptr.shape[0] - 1), C.c_int32(1 if accumulate else 0), B._ptr(energy), B._ptr(saved),
        C.c_size_t(saved.numel()), B._ptr(scratch), C.c_size_t(scratch.numel())))
    return energy


def gp_output_backward(ctx, w, m, rbf, dst, graph_ptr, n_atoms, grad_energy, saved, accumulate_grad_m, grad_m, grad_w,
                       scratch):
    emb, out_emb, R, L = _shape(w)
    ws = _out(w)
    gws = _out(grad_w) if grad_w is not None else None
    ctx.check(B.load().gp_output_backward(
        ctx._h, C.c_int32(emb), C.c_int32(out_emb), C.c_int32(R), C.c_int32(L), C.byref(ws), B._ptr(m), B._ptr(rbf),
        B._ptr(dst), B._ptr(graph_ptr), C.c_int64(n_atoms), C.c_int64(m.shape[0]), C.c_int32(graph_ptr.shape[0] - 1),
        B._ptr(grad_energy), B._ptr(saved), C.c_size_t(saved.numel()), C.c_int32(1 if accumulate_grad_m else 0),
        B._ptr(grad_m), C.byref(gws) if gws is not None else None, B._ptr(scratch), C.c_size_t(scratch.numel())))
    return grad_m


class ModelD:
    """Variant-D interaction blocks, each followed by an output block; the structure energies are the
    sums of the output blocks' contributions.  forward(m0) -> energy[n_graphs];
    backward(grad_energy) -> (grad m0, block weight gradients, output-block weight gradients)."""

    def __init__(self, ctx, dims, block_weights, out_weights, edges, trip, basis, graph_ptr):
        assert len(block_weights) == len(out_weights)
        self.ctx, self.dims, self.edges, self.trip, self.basis, self.graph_ptr = ctx, dims, edges, trip, basis, graph_ptr
        self.wb, self.wo = block_weights, out_weights
        self.n_blocks = len(block_weights)
        dev = ctx.device
        E, T, N = trip["n_edges"], trip["n_triplets"], edges["n_atoms"]
        sb, cb = B.gp_block_workspace(dims, E, T)
        emb, out_emb, R, L = _shape(out_weights[0])
        so, co = gp_output_workspace(emb, out_emb, R, L, N, E)
        u8 = lambda n: torch.empty(max(n, 8), dtype=torch.uint8, device=dev)
        self.saved_b = [u8(sb) for _ in range(self.n_blocks)]
        self.saved_o = [u8(so) for _ in range(self.n_blocks)]
        self.scratch_b, self.scratch_o = u8(cb), u8(co)
        self.m = [torch.empty((E, dims.emb), dtype=torch.float32, device=dev) for _ in range(self.n_blocks)]
        self.g = [torch.empty((E, dims.emb), dtype=torch.float32, device=dev) for _ in range(2)]
        self.energy = torch.empty(graph_ptr.shape[0] - 1, dtype=torch.float32, device=dev)
        self.grad_wb = [{k: torch.empty_like(v) for k, v in w.items()} for w in block_weights]
        self.grad_wo = [{k: torch.empty_like(v) for k, v in w.items()} for w in out_weights]
        self.m_in = None

    def forward(self, m0):
        self.m_in = m0
        cur = m0
        for b in range(self.n_blocks):
            B.gp_block_forward_D(self.ctx, self.dims, self.wb[b], self.trip, self.basis, cur, self.m[b], self.saved_b[b],
                                 self.scratch_b)
            cur = self.m[b]
            gp_output_forward(self.ctx, self.wo[b], cur, self.basis["rbf"], self.edges["row_ptr"], self.graph_ptr,
                              b > 0, self.energy, self.saved_o[b], self.scratch_o)
        return self.energy

    def backward(self, grad_energy):
        N = self.edges["n_atoms"]
        g = None
        for b in reversed(range(self.n_blocks)):
            # gradient w.r.t. this block's output: what the next block passed down (if any) plus this output block's
            tot = self.g[b % 2] if g is None else g
            gp_output_backward(self.ctx, self.wo[b], self.m[b], self.basis["rbf"], self.edges["dst"], self.graph_ptr, N,
                               grad_energy, self.saved_o[b], g is not None, tot, self.grad_wo[b], self.scratch_o)
            m_in = self.m_in if b == 0 else self.m[b - 1]
            out = self.g[(b + 1) % 2]
            B.gp_block_backward_D(self.ctx, self.dims, self.wb[b], self.trip, self.basis, m_in, self.saved_b[b], tot, out,
                                  self.grad_wb[b], self.scratch_b)
            g = out
        return g, self.grad_wb, self.grad_wo
