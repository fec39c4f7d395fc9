"""Seeded random tensors: edge embeddings, upstream gradients, layer weights.

Weights are stored as W[in, out] (a layer computes x @ W + b), fp32, drawn
Glorot-uniform U(-a, a) with a = sqrt(6 / (fan_in + fan_out)) in the fixed
order listed in each function.  Biases are zero unless bias_scale > 0, in
which case they are U(-bias_scale, bias_scale) so that tests exercise them.
"""
import numpy as np


def glorot(rng, shape, fan_in=None, fan_out=None):
    fan_in = shape[0] if fan_in is None else fan_in
    fan_out = shape[-1] if fan_out is None else fan_out
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, size=shape).astype(np.float32)


def _bias(rng, n, bias_scale):
    if bias_scale > 0:
        return rng.uniform(-bias_scale, bias_scale, size=n).astype(np.float32)
    return np.zeros(n, dtype=np.float32)


def weights_D(dims, seed=0, bias_scale=0.0):
    """Weights of one Hadamard-interaction block (variant D) as an ordered dict."""
    rng = np.random.default_rng(seed)
    e, i, b = dims.emb, dims.int_emb, dims.basis_emb
    R, S = dims.num_radial, dims.num_spherical
    w = {}
    w["W_ji"] = glorot(rng, (e, e)); w["b_ji"] = _bias(rng, e, bias_scale)
    w["W_kj"] = glorot(rng, (e, e)); w["b_kj"] = _bias(rng, e, bias_scale)
    w["W_rbf1"] = glorot(rng, (R, b))
    w["W_rbf2"] = glorot(rng, (b, e))
    w["W_down"] = glorot(rng, (e, i))
    w["W_sbf1"] = glorot(rng, (S * R, b))
    w["W_sbf2"] = glorot(rng, (b, i))
    w["W_up"] = glorot(rng, (i, e))
    for r in range(dims.n_res_before):
        w[f"W_b{r}_1"] = glorot(rng, (e, e)); w[f"b_b{r}_1"] = _bias(rng, e, bias_scale)
        w[f"W_b{r}_2"] = glorot(rng, (e, e)); w[f"b_b{r}_2"] = _bias(rng, e, bias_scale)
    w["W_lin"] = glorot(rng, (e, e)); w["b_lin"] = _bias(rng, e, bias_scale)
    for r in range(dims.n_res_after):
        w[f"W_a{r}_1"] = glorot(rng, (e, e)); w[f"b_a{r}_1"] = _bias(rng, e, bias_scale)
        w[f"W_a{r}_2"] = glorot(rng, (e, e)); w[f"b_a{r}_2"] = _bias(rng, e, bias_scale)
    return w


def weights_G(dims, seed=0):
    """Weights of one bilinear-interaction block (variant G) as an ordered dict."""
    rng = np.random.default_rng(seed)
    e, t = dims.emb, dims.int_emb
    R, S = dims.num_radial, dims.num_spherical
    w = {}
    w["W_ba"] = glorot(rng, (e, e))
    w["W_rbfS"] = glorot(rng, (R, dims.emb_rbf))
    w["W_rbfB"] = glorot(rng, (dims.emb_rbf, e))
    w["W_down"] = glorot(rng, (e, t))
    w["W_c"] = glorot(rng, (S, R, dims.emb_cbf), fan_in=R, fan_out=dims.emb_cbf)
    w["W_bil"] = glorot(rng, (dims.emb_cbf, t, dims.emb_bil),
                        fan_in=dims.emb_cbf * t, fan_out=dims.emb_bil)
    w["W_up"] = glorot(rng, (dims.emb_bil, e))
    w["W_skip"] = glorot(rng, (e, e))
    if getattr(dims, "symmetric", False):
        w["W_up_ac"] = glorot(rng, (dims.emb_bil, e))
    return w


def weights_head(emb, hidden, seed=0, bias_scale=0.0):
    """Per-atom energy head: E_i = w2 . act(h_i W1 + b1) + b2."""
    rng = np.random.default_rng(seed)
    w = {}
    w["W1"] = glorot(rng, (emb, hidden)); w["b1"] = _bias(rng, hidden, bias_scale)
    w["w2"] = glorot(rng, (hidden, 1)).reshape(hidden); w["b2"] = _bias(rng, 1, bias_scale)
    return w


def weights_out(emb, out_emb, num_radial, n_layers=3, seed=0, bias_scale=0.0):
    """Output block: radial weighting of the messages, up-projection, n_layers dense layers, final vector."""
    rng = np.random.default_rng(seed)
    w = {}
    w["W_rbf"] = glorot(rng, (num_radial, emb))
    w["W_up"] = glorot(rng, (emb, out_emb))
    for k in range(n_layers):
        w[f"W{k}"] = glorot(rng, (out_emb, out_emb)); w[f"b{k}"] = _bias(rng, out_emb, bias_scale)
    w["w_final"] = glorot(rng, (out_emb, 1)).reshape(out_emb)
    return w


def edge_embeddings(n_edges, emb, seed=0):
    """Input messages m ~ N(0,1) and an upstream gradient of the same shape."""
    rng = np.random.default_rng(seed)
    m = rng.standard_normal((n_edges, emb)).astype(np.float32)
    g = rng.standard_normal((n_edges, emb)).astype(np.float32)
    return m, g
