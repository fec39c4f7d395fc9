"""Buffer management for a stack of interaction blocks (allocation and call sequencing only)."""
import torch

from . import binding as B


class StackD:
    """n_blocks variant-D blocks sharing one graph and one basis.

    All device buffers (saved activations per block, scratch, intermediate messages and
    gradients) are allocated once; forward()/backward() only issue library calls.
    """

    def __init__(self, ctx, dims, weights_list, trip, basis):
        self.ctx, self.dims, self.trip, self.basis = ctx, dims, trip, basis
        self.w = weights_list
        self.n_blocks = len(weights_list)
        E, T = trip["n_edges"], trip["n_triplets"]
        self.E = E
        saved_b, scratch_b = B.gp_block_workspace(dims, E, T)
        dev = ctx.device
        self.saved = [torch.empty(max(saved_b, 8), dtype=torch.uint8, device=dev) for _ in range(self.n_blocks)]
        self.scratch = torch.empty(max(scratch_b, 8), dtype=torch.uint8, device=dev)
        self.m = [torch.empty((E, dims.emb), dtype=torch.float32, device=dev) for _ in range(self.n_blocks)]
        self.g = [torch.empty((E, dims.emb), dtype=torch.float32, device=dev) for _ in range(2)]
        self.grad_w = [{k: torch.empty_like(v) for k, v in w.items()} for w in weights_list]
        self.m_in = None

    def forward(self, m_in):
        self.m_in = m_in
        cur = m_in
        for b in range(self.n_blocks):
            B.gp_block_forward_D(self.ctx, self.dims, self.w[b], self.trip, self.basis, cur, self.m[b],
                                 self.saved[b], self.scratch)
            cur = self.m[b]
        return cur

    def backward(self, grad_out, basis_grads=None):
        """basis_grads: dict with any of 'grad_rbf' [E, R], 'grad_rad' [E, S * R], 'grad_cos_kj' [T] (fp32 device
        tensors): the blocks' gradients with respect to the basis are summed into them."""
        g = grad_out
        for b in reversed(range(self.n_blocks)):
            m_in = self.m_in if b == 0 else self.m[b - 1]
            out = self.g[b % 2]
            if basis_grads is None:
                B.gp_block_backward_D(self.ctx, self.dims, self.w[b], self.trip, self.basis, m_in, self.saved[b], g, out,
                                      self.grad_w[b], self.scratch)
            else:
                B.gp_block_backward_D_basis(self.ctx, self.dims, self.w[b], self.trip, self.basis, m_in, self.saved[b], g, out,
                                            self.grad_w[b], self.scratch, basis_grads.get("grad_rbf"),
                                            basis_grads.get("grad_rad"), basis_grads.get("grad_cos_kj"),
                                            accumulate=b != self.n_blocks - 1)
            g = out
        return g, self.grad_w
