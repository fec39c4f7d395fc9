"""ctypes binding of the energy head, the out-edge lists and the force assembly."""
import ctypes as C

import torch

from . import binding as B
from .binding_g import StackG

__all__ = ["gp_energy_workspace", "gp_energy_forward", "gp_energy_backward", "gp_edges_by_source",
           "gp_forces_from_basis_grad", "gp_forces_from_basis_grad_D", "ForceModelG", "ForceModelD"]


class _WeightsHead(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("W1", "b1", "w2", "b2")]


def _head(w):
    return _WeightsHead(W1=B._ptr(w["W1"]), b1=B._ptr(w["b1"]), w2=B._ptr(w["w2"]), b2=B._ptr(w["b2"]))


def gp_energy_workspace(emb, hidden, n_atoms):
    a, b = C.c_size_t(), C.c_size_t()
    rc = B.load().gp_energy_workspace(C.c_int32(emb), C.c_int32(hidden), C.c_int64(n_atoms), C.byref(a), C.byref(b))
    if rc != 0:
        raise B.GpError(rc, "gp_energy_workspace")
    return a.value, b.value


def gp_energy_forward(ctx, emb, hidden, w, m, row_ptr, graph_ptr, energy, saved):
    h = _head(w)
    ctx.check(B.load().gp_energy_forward(ctx._h, C.c_int32(emb), C.c_int32(hidden), C.byref(h), B._ptr(m), B._ptr(row_ptr),
                                         B._ptr(graph_ptr), C.c_int64(row_ptr.shape[0] - 1),
                                         C.c_int32(graph_ptr.shape[0] - 1), B._ptr(energy), B._ptr(saved),
                                         C.c_size_t(saved.numel())))
    return energy


def gp_energy_backward(ctx, emb, hidden, w, dst, n_atoms, saved, grad_m, grad_w, scratch):
    h = _head(w)
    gh = _head(grad_w) if grad_w is not None else None
    ctx.check(B.load().gp_energy_backward(ctx._h, C.c_int32(emb), C.c_int32(hidden), C.byref(h), B._ptr(dst),
                                          C.c_int64(n_atoms), C.c_int64(dst.shape[0]), B._ptr(saved),
                                          C.c_size_t(saved.numel()), B._ptr(grad_m),
                                          C.byref(gh) if gh is not None else None, B._ptr(scratch),
                                          C.c_size_t(scratch.numel())))
    return grad_m


gp_edges_by_source = B.gp_edges_by_source


def gp_forces_from_basis_grad(ctx, dims, edges, trip, out_ptr, out_list, grad_rbf, grad_cos_kj, forces, ws):
    d, g = B.Dims(dims), B.Graph(trip)
    ctx.check(B.load().gp_forces_from_basis_grad(
        ctx._h, C.byref(d), C.byref(g), B._ptr(trip["perm_kj"]), B._ptr(edges["row_ptr"]), B._ptr(out_ptr),
        B._ptr(out_list), C.c_int64(edges["n_atoms"]), B._ptr(edges["dist"]), B._ptr(edges["unit"]), B._ptr(grad_rbf),
        B._ptr(grad_cos_kj), B._ptr(forces), B._ptr(ws), C.c_size_t(ws.numel())))
    return forces


def gp_forces_from_basis_grad_D(ctx, dims, edges, trip, out_ptr, out_list, grad_rbf, grad_rad, grad_cos_kj, forces, ws):
    d, g = B.Dims(dims), B.Graph(trip)
    ctx.check(B.load().gp_forces_from_basis_grad_D(
        ctx._h, C.byref(d), C.byref(g), B._ptr(trip["perm_kj"]), B._ptr(edges["row_ptr"]), B._ptr(out_ptr),
        B._ptr(out_list), C.c_int64(edges["n_atoms"]), B._ptr(edges["dist"]), B._ptr(edges["unit"]), B._ptr(grad_rbf),
        B._ptr(grad_rad), B._ptr(grad_cos_kj), B._ptr(forces), B._ptr(ws), C.c_size_t(ws.numel())))
    return forces


class ForceModelD:
    """Variant-D block stack + energy head; energy_and_forces() runs forward, backward and the position-gradient
    assembly.  Allocation and call sequencing only."""

    def __init__(self, ctx, dims, weights_list, head_w, hidden, edges, trip, basis, graph_ptr):
        from .stack import StackD
        self.ctx, self.dims, self.edges, self.trip, self.basis = ctx, dims, edges, trip, basis
        self.stack = StackD(ctx, dims, weights_list, trip, basis)
        self.head_w, self.hidden, self.graph_ptr = head_w, hidden, graph_ptr
        dev = ctx.device
        N, E, T = edges["n_atoms"], edges["n_edges"], trip["n_triplets"]
        sb, cb = gp_energy_workspace(dims.emb, hidden, N)
        self.h_saved = torch.empty(max(sb, 8), dtype=torch.uint8, device=dev)
        self.h_scratch = torch.empty(max(cb, 8), dtype=torch.uint8, device=dev)
        self.energy = torch.empty(graph_ptr.shape[0] - 1, dtype=torch.float32, device=dev)
        self.grad_m = torch.empty((E, dims.emb), dtype=torch.float32, device=dev)
        self.basis_grads = {"grad_rbf": torch.empty((E, dims.num_radial), dtype=torch.float32, device=dev),
                            "grad_rad": torch.empty((E, dims.num_spherical * dims.num_radial), dtype=torch.float32, device=dev),
                            "grad_cos_kj": torch.empty(max(T, 1), dtype=torch.float32, device=dev)}
        self.forces = torch.empty((N, 3), dtype=torch.float32, device=dev)
        self.out_ptr, self.out_list = gp_edges_by_source(ctx, edges)
        nb = C.c_size_t()
        ctx.check(B.load().gp_forces_workspace(C.c_int64(E), C.c_int64(T), C.byref(nb)))
        self.f_ws = torch.empty(max(nb.value, 8), dtype=torch.uint8, device=dev)
        self.head_grad = {k: torch.empty_like(v) for k, v in head_w.items()}

    def energy_and_forces(self, m0):
        d = self.dims
        m = self.stack.forward(m0)
        gp_energy_forward(self.ctx, d.emb, self.hidden, self.head_w, m, self.edges["row_ptr"], self.graph_ptr, self.energy,
                          self.h_saved)
        gp_energy_backward(self.ctx, d.emb, self.hidden, self.head_w, self.edges["dst"], self.edges["n_atoms"],
                           self.h_saved, self.grad_m, self.head_grad, self.h_scratch)
        self.stack.backward(self.grad_m, basis_grads=self.basis_grads)
        bg = self.basis_grads
        gp_forces_from_basis_grad_D(self.ctx, d, self.edges, self.trip, self.out_ptr, self.out_list, bg["grad_rbf"],
                                    bg["grad_rad"], bg["grad_cos_kj"], self.forces, self.f_ws)
        return self.energy, self.forces


class ForceModelG:
    """Variant-G block stack + energy head; energy_and_forces() runs forward, backward and the
    position-gradient assembly.  Allocation and call sequencing only."""

    def __init__(self, ctx, dims, weights_list, head_w, hidden, edges, trip, basis, graph_ptr):
        self.ctx, self.dims, self.edges, self.trip, self.basis = ctx, dims, edges, trip, basis
        self.stack = StackG(ctx, dims, weights_list, trip, basis)
        self.head_w, self.hidden, self.graph_ptr = head_w, hidden, graph_ptr
        dev = ctx.device
        N, E, T = edges["n_atoms"], edges["n_edges"], trip["n_triplets"]
        sb, cb = gp_energy_workspace(dims.emb, hidden, N)
        self.h_saved = torch.empty(max(sb, 8), dtype=torch.uint8, device=dev)
        self.h_scratch = torch.empty(max(cb, 8), dtype=torch.uint8, device=dev)
        self.energy = torch.empty(graph_ptr.shape[0] - 1, dtype=torch.float32, device=dev)
        self.grad_m = torch.empty((E, dims.emb), dtype=torch.float32, device=dev)
        self.grad_rbf = torch.empty((E, dims.num_radial), dtype=torch.float32, device=dev)
        self.grad_cos_kj = torch.empty(T, dtype=torch.float32, device=dev)
        self.forces = torch.empty((N, 3), dtype=torch.float32, device=dev)
        self.out_ptr, self.out_list = gp_edges_by_source(ctx, edges)
        nb = C.c_size_t()
        ctx.check(B.load().gp_forces_workspace(C.c_int64(E), C.c_int64(T), C.byref(nb)))
        self.f_ws = torch.empty(max(nb.value, 8), dtype=torch.uint8, device=dev)
        self.head_grad = {k: torch.empty_like(v) for k, v in head_w.items()}

    def energy_and_forces(self, m0):
        d = self.dims
        m = self.stack.forward(m0)
        gp_energy_forward(self.ctx, d.emb, self.hidden, self.head_w, m, self.edges["row_ptr"], self.graph_ptr, self.energy,
                          self.h_saved)
        gp_energy_backward(self.ctx, d.emb, self.hidden, self.head_w, self.edges["dst"], self.edges["n_atoms"],
                           self.h_saved, self.grad_m, self.head_grad, self.h_scratch)
        self.stack.backward(self.grad_m, grad_rbf=self.grad_rbf, grad_cos_kj=self.grad_cos_kj)
        gp_forces_from_basis_grad(self.ctx, d, self.edges, self.trip, self.out_ptr, self.out_list, self.grad_rbf,
                                  self.grad_cos_kj, self.forces, self.f_ws)
        return self.energy, self.forces
