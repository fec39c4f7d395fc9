"""ctypes binding of the variant-G (bilinear) block entry points."""
import ctypes as C

import torch

from . import binding as B

__all__ = ["G_WEIGHT_NAMES", "gp_block_forward_G", "gp_block_backward_G", "gp_block_G_stacks_bf16", "StackG"]

G_WEIGHT_NAMES = ("W_ba", "W_rbfS", "W_rbfB", "W_down", "W_c", "W_bil", "W_up", "W_skip", "W_up_ac")


class _WeightsG(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in G_WEIGHT_NAMES]


def _weights_G(w):
    s = _WeightsG()
    for n in G_WEIGHT_NAMES:
        setattr(s, n, B._ptr(w.get(n)))     # W_up_ac exists only for symmetric blocks
    return s


def gp_block_G_stacks_bf16(dims):
    d = B.Dims(dims)
    return bool(B.load().gp_block_G_stacks_bf16(C.byref(d)))


def _is_bf16(t):
    return t.dtype == torch.bfloat16


def gp_block_forward_G(ctx, dims, w, trip, basis, m_in, m_out, saved, scratch):
    """m_in / m_out fp32, or bf16 tensors: then gp_block_forward_G_stacked is called with the matching flags."""
    lib = B.load()
    d, g, b, ws = B.Dims(dims), B.Graph(trip), B.Basis(basis), _weights_G(w)
    if _is_bf16(m_in) or _is_bf16(m_out):
        ctx.check(lib.gp_block_forward_G_stacked(ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), B._ptr(m_in),
                                                 C.c_int32(_is_bf16(m_in)), B._ptr(m_out), C.c_int32(_is_bf16(m_out)),
                                                 B._ptr(saved), C.c_size_t(saved.numel()), B._ptr(scratch),
                                                 C.c_size_t(scratch.numel())))
        return m_out
    ctx.check(lib.gp_block_forward_G(ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), B._ptr(m_in),
                                     B._ptr(m_out), B._ptr(saved), C.c_size_t(saved.numel()), B._ptr(scratch),
                                     C.c_size_t(scratch.numel())))
    return m_out


def gp_block_backward_G(ctx, dims, w, trip, basis, m_in, saved, grad_m_out, grad_m_in, grad_w, scratch, grad_rbf=None,
                        grad_cos_kj=None, accumulate=False):
    """m_in, grad_m_out, grad_m_in fp32, or bf16 tensors (gp_block_backward_G_stacked with the matching flags)."""
    lib = B.load()
    d, g, b = B.Dims(dims), B.Graph(trip), B.Basis(basis)
    ws, gws = _weights_G(w), _weights_G(grad_w)
    if _is_bf16(m_in) or _is_bf16(grad_m_out) or _is_bf16(grad_m_in):
        ctx.check(lib.gp_block_backward_G_stacked(
            ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), B._ptr(m_in), C.c_int32(_is_bf16(m_in)), B._ptr(saved),
            C.c_size_t(saved.numel()), B._ptr(grad_m_out), C.c_int32(_is_bf16(grad_m_out)), B._ptr(grad_m_in),
            C.c_int32(_is_bf16(grad_m_in)), C.byref(gws), B._ptr(grad_rbf), B._ptr(grad_cos_kj),
            C.c_int32(1 if accumulate else 0), B._ptr(scratch), C.c_size_t(scratch.numel())))
        return grad_m_in, grad_w
    ctx.check(lib.gp_block_backward_G(ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), B._ptr(m_in),
                                      B._ptr(saved), C.c_size_t(saved.numel()), B._ptr(grad_m_out), B._ptr(grad_m_in),
                                      C.byref(gws), B._ptr(grad_rbf), B._ptr(grad_cos_kj), C.c_int32(1 if accumulate else 0),
                                      B._ptr(scratch), C.c_size_t(scratch.numel())))
    return grad_m_in, grad_w


class StackG:
    """n_blocks variant-G blocks sharing one graph and one basis (buffers allocated once).  Between bf16 blocks the
    messages, and for non-symmetric blocks the gradients, are handed over as bf16 (gp_block_*_G_stacked)."""

    def __init__(self, ctx, dims, weights_list, trip, basis, handoff_bf16=True):
        self.ctx, self.dims, self.trip, self.basis = ctx, dims, trip, basis
        self.w = weights_list
        self.n_blocks = len(weights_list)
        E, T = trip["n_edges"], trip["n_triplets"]
        saved_b, scratch_b = B.gp_block_workspace(dims, E, T, trip.get("n_atoms", 0) if trip.get("out_list") is not None else 0)
        dev = ctx.device
        self.saved = [torch.empty(max(saved_b, 8), dtype=torch.uint8, device=dev) for _ in range(self.n_blocks)]
        self.scratch = torch.empty(max(scratch_b, 8), dtype=torch.uint8, device=dev)
        self.half_m = bool(handoff_bf16) and self.n_blocks > 1 and gp_block_G_stacks_bf16(dims)
        self.half_g = self.half_m and not getattr(dims, "symmetric", False)
        # outputs of the blocks: the last one fp32 (the caller's), the inner ones bf16 when handed over so
        self.m = [torch.empty((E, dims.emb), dtype=torch.bfloat16 if self.half_m and b < self.n_blocks - 1 else torch.float32,
                              device=dev) for b in range(self.n_blocks)]
        self.g = [torch.empty((E, dims.emb), dtype=torch.float32, device=dev) for _ in range(2)]
        self.gh = [torch.empty((E, dims.emb), dtype=torch.bfloat16, device=dev) for _ in range(2)] if self.half_g else None
        self.grad_w = [{k: torch.empty_like(v) for k, v in w.items()} for w in weights_list]
        self.m_in = None

    def forward(self, m_in):
        self.m_in = m_in
        cur = m_in
        for b in range(self.n_blocks):
            gp_block_forward_G(self.ctx, self.dims, self.w[b], self.trip, self.basis, cur, self.m[b], self.saved[b],
                               self.scratch)
            cur = self.m[b]
        return cur

    def backward(self, grad_out, grad_rbf=None, grad_cos_kj=None):
        """grad_rbf [E,R] / grad_cos_kj [T], if given, receive the basis gradients summed over all blocks
        (the first block processed overwrites, the others accumulate inside the library)."""
        g = grad_out
        first = True
        for b in reversed(range(self.n_blocks)):
            m_in = self.m_in if b == 0 else self.m[b - 1]
            out = self.gh[b % 2] if self.half_g and b > 0 else self.g[b % 2]
            gp_block_backward_G(self.ctx, self.dims, self.w[b], self.trip, self.basis, m_in, self.saved[b], g, out,
                                self.grad_w[b], self.scratch, grad_rbf, grad_cos_kj, accumulate=not first)
            g = out
            first = False
        return g, self.grad_w
