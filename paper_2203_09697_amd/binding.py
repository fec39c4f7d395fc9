"""ctypes binding of libgpgnn.so: same names as the C ABI, tensors in, tensors out."""
import ctypes as C
import os

import torch

__all__ = [
    "GpError", "load", "library_path", "Context", "Dims", "Graph", "Basis",
    "gp_version", "gp_deferred_status", "gp_profile_enable", "gp_profile_reset", "gp_profile_collect", "gp_set_side_stream", "gp_set_triplet_mfma", "gp_set_f32_gemm",
    "gp_measure_peaks", "gp_edges_by_source", "gp_edges_by_source_static", "gp_reverse_edges", "gp_edges", "gp_triplets", "gp_basis_forward", "gp_block_workspace",
    "gp_block_forward_D", "gp_block_backward_D", "gp_block_backward_D_basis", "gp_triplet_aggregate_fwd",
    "gp_triplet_aggregate_bwd", "gp_linear_forward", "build_graph", "weights_to_device",
    "TRIPLET_STREAM", "TRIPLET_PER_EDGE", "TRIPLET_PER_ATOM", "TRIPLET_PER_ATOM_TWO_KERNELS", "gp_triplet_workspace",
    "gp_triplet_hadamard_fwd", "gp_triplet_hadamard_bwd", "gp_triplet_bilinear_fwd", "gp_triplet_bilinear_bwd_H",
    "gp_triplet_bilinear_grad_cos",
    "EXPORTED_SYMBOLS", "D_WEIGHT_ORDER",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

GP_MAX_RES = 4
STATUS = {0: "GP_OK", -1: "GP_BAD_ARG", -2: "GP_BUFFER_TOO_SMALL", -3: "GP_INT32_OVERFLOW",
          -4: "GP_HIP_ERROR", -5: "GP_UNSUPPORTED_DIMS"}

EXPORTED_SYMBOLS = [
    "gp_create", "gp_destroy", "gp_last_error", "gp_version",
    "gp_profile_enable", "gp_profile_reset", "gp_profile_count", "gp_profile_get", "gp_set_side_stream", "gp_set_triplet_mfma", "gp_set_f32_gemm", "gp_deferred_status", "gp_measure_peaks",
    "gp_edges_workspace", "gp_edges_count", "gp_edges_fill", "gp_edges_count_pbc", "gp_edges_fill_pbc",
    "gp_triplets_count_pbc", "gp_triplets_fill_pbc",
    "gp_triplets_workspace", "gp_triplets_count", "gp_triplets_fill", "gp_csr_max_degree", "gp_reverse_edges",
    "gp_basis_forward", "gp_block_workspace", "gp_block_forward_D", "gp_block_backward_D", "gp_block_backward_D_basis",
    "gp_block_forward_G", "gp_block_backward_G", "gp_block_G_stacks_bf16", "gp_block_forward_G_stacked", "gp_block_backward_G_stacked",
    "gp_energy_workspace", "gp_energy_forward", "gp_energy_backward",
    "gp_output_workspace", "gp_output_forward", "gp_output_backward",
    "gp_edges_by_source_workspace", "gp_edges_by_source", "gp_edges_by_source_static", "gp_forces_workspace", "gp_forces_from_basis_grad", "gp_forces_from_basis_grad_D",
    "gp_triplet_aggregate_fwd", "gp_triplet_aggregate_bwd", "gp_linear_forward", "gp_linear_forward_bf16",
    "gp_triplet_workspace", "gp_triplet_hadamard_fwd", "gp_triplet_hadamard_bwd", "gp_triplet_bilinear_fwd",
    "gp_triplet_bilinear_bwd_H", "gp_triplet_bilinear_grad_cos",
]


class GpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s (%d): %s" % (STATUS.get(code, "?"), code, msg))
        self.code = code


def library_path():
    return os.path.join(_HERE, "libgpgnn.so")


def load():
    """Loads the HIP library; raises if it has not been built (there is no fallback)."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError("%s not found: build it with `python -m paper_2203_09697_amd.build`" % path)
        lib = C.CDLL(path)
        lib.gp_last_error.restype = C.c_char_p
        lib.gp_version.restype = C.c_char_p
        lib.gp_destroy.restype = None
        _LIB = lib
    return _LIB


# ------------------------------------------------------------------ C structs
class _Dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "variant", "dtype", "emb", "int_emb", "basis_emb", "emb_rbf", "emb_cbf", "emb_bil",
        "num_radial", "num_spherical", "envelope_p", "n_res_before", "n_res_after", "symmetric", "radial_at_target")] + [("cutoff", C.c_float)]


class _Graph(C.Structure):
    _fields_ = [("n_edges", C.c_int64), ("n_triplets", C.c_int64), ("idx_kj", C.c_void_p),
                ("seg_ptr_ji", C.c_void_p), ("idx_ji_kj", C.c_void_p), ("seg_ptr_kj", C.c_void_p),
                ("n_atoms", C.c_int64), ("max_in_degree", C.c_int32), ("max_out_degree", C.c_int32),
                ("row_ptr", C.c_void_p), ("out_ptr", C.c_void_p), ("out_list", C.c_void_p), ("perm_kj", C.c_void_p), ("id_swap", C.c_void_p)]


class _Basis(C.Structure):
    _fields_ = [("rbf", C.c_void_p), ("rad", C.c_void_p), ("cos_alpha", C.c_void_p), ("cos_alpha_kj", C.c_void_p)]


class _WeightsD(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "W_ji", "b_ji", "W_kj", "b_kj", "W_rbf1", "W_rbf2", "W_down", "W_sbf1", "W_sbf2", "W_up")] + [
        ("res_before", (C.c_void_p * 4) * GP_MAX_RES), ("W_lin", C.c_void_p), ("b_lin", C.c_void_p),
        ("res_after", (C.c_void_p * 4) * GP_MAX_RES)]


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    return C.c_void_p(t.data_ptr())


def Dims(d):
    """gp_dims from a synth.BlockDims-like object (attribute access only)."""
    return _Dims(variant=0 if d.variant == "D" else 1, dtype=0 if d.dtype == "f32" else 1, emb=d.emb,
                 int_emb=d.int_emb, basis_emb=d.basis_emb, emb_rbf=d.emb_rbf, emb_cbf=d.emb_cbf,
                 emb_bil=d.emb_bil, num_radial=d.num_radial, num_spherical=d.num_spherical,
                 envelope_p=d.envelope_p, n_res_before=d.n_res_before, n_res_after=d.n_res_after,
                 symmetric=1 if getattr(d, "symmetric", False) else 0,
                 radial_at_target=1 if getattr(d, "radial_at_target", False) else 0, cutoff=d.cutoff)


def Graph(g):
    """gp_graph from the dict returned by build_graph / gp_triplets."""
    return _Graph(n_edges=g["n_edges"], n_triplets=g["n_triplets"], idx_kj=_ptr(g["idx_kj"]),
                  seg_ptr_ji=_ptr(g["seg_ptr_ji"]), idx_ji_kj=_ptr(g.get("idx_ji_kj")),
                  seg_ptr_kj=_ptr(g.get("seg_ptr_kj")),
                  n_atoms=g.get("n_atoms", 0) if g.get("out_list") is not None else 0,
                  max_in_degree=g.get("max_in_degree", 0), max_out_degree=g.get("max_out_degree", 0), row_ptr=_ptr(g.get("row_ptr")),
                  out_ptr=_ptr(g.get("out_ptr")), out_list=_ptr(g.get("out_list")), perm_kj=_ptr(g.get("perm_kj")), id_swap=_ptr(g.get("id_swap")))


def Basis(b):
    return _Basis(rbf=_ptr(b.get("rbf")), rad=_ptr(b.get("rad")), cos_alpha=_ptr(b.get("cos_alpha")),
                  cos_alpha_kj=_ptr(b.get("cos_alpha_kj")))


def D_WEIGHT_ORDER(dims):
    names = ["W_ji", "b_ji", "W_kj", "b_kj", "W_rbf1", "W_rbf2", "W_down", "W_sbf1", "W_sbf2", "W_up"]
    for r in range(dims.n_res_before):
        names += [f"W_b{r}_1", f"b_b{r}_1", f"W_b{r}_2", f"b_b{r}_2"]
    names += ["W_lin", "b_lin"]
    for r in range(dims.n_res_after):
        names += [f"W_a{r}_1", f"b_a{r}_1", f"W_a{r}_2", f"b_a{r}_2"]
    return names


def _weights_D(dims, w):
    s = _WeightsD()
    for n in ("W_ji", "b_ji", "W_kj", "b_kj", "W_rbf1", "W_rbf2", "W_down", "W_sbf1", "W_sbf2", "W_up", "W_lin", "b_lin"):
        setattr(s, n, _ptr(w[n]))
    for r in range(dims.n_res_before):
        for q, n in enumerate((f"W_b{r}_1", f"b_b{r}_1", f"W_b{r}_2", f"b_b{r}_2")):
            s.res_before[r][q] = w[n].data_ptr()
    for r in range(dims.n_res_after):
        for q, n in enumerate((f"W_a{r}_1", f"b_a{r}_1", f"W_a{r}_2", f"b_a{r}_2")):
            s.res_after[r][q] = w[n].data_ptr()
    return s


def weights_to_device(w, device="cuda:0"):
    """dict of numpy arrays -> dict of fp32 device tensors."""
    return {k: torch.as_tensor(v, dtype=torch.float32).contiguous().to(device) for k, v in w.items()}


# ------------------------------------------------------------------ context
class Context:
    """gp_ctx bound to a device and to torch's current stream on it (or a given stream)."""

    def __init__(self, device_id=0, stream=None):
        lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("gpgnn needs a GPU: torch.cuda.is_available() is False")
        self.device = torch.device("cuda", device_id)
        st = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.stream = st
        self._h = C.c_void_p()
        rc = lib.gp_create(C.byref(self._h), C.c_int(device_id), C.c_void_p(st.cuda_stream))
        if rc != 0:
            raise GpError(rc, "gp_create failed")

    def check(self, rc):
        if rc != 0:
            raise GpError(rc, load().gp_last_error(self._h).decode())

    def close(self):
        if self._h:
            load().gp_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gp_version():
    return load().gp_version().decode()


def gp_profile_enable(ctx, on):
    ctx.check(load().gp_profile_enable(ctx._h, C.c_int(1 if on else 0)))


def gp_measure_peaks(ctx, mib=512):
    """{"copy_GBps", "mfma_f32_TFLOPs", "mfma_bf16_TFLOPs"} measured on the context's device."""
    ws = torch.empty(mib << 20, dtype=torch.uint8, device=ctx.device)
    a, b, c = C.c_double(), C.c_double(), C.c_double()
    ctx.check(load().gp_measure_peaks(ctx._h, _ptr(ws), C.c_size_t(ws.numel()), C.byref(a), C.byref(b), C.byref(c)))
    return {"copy_GBps": a.value, "mfma_f32_TFLOPs": b.value, "mfma_bf16_TFLOPs": c.value}


def gp_set_triplet_mfma(ctx, mode):
    ctx.check(load().gp_set_triplet_mfma(ctx._h, C.c_int(mode)))


def gp_set_f32_gemm(ctx, split):
    ctx.check(load().gp_set_f32_gemm(ctx._h, C.c_int(1 if split else 0)))


def gp_deferred_status(ctx):
    """Synchronises the context's stream and raises for errors that only a kernel could detect."""
    ctx.check(load().gp_deferred_status(ctx._h))


def gp_set_side_stream(ctx, on):
    ctx.check(load().gp_set_side_stream(ctx._h, C.c_int(1 if on else 0)))


def gp_profile_reset(ctx):
    ctx.check(load().gp_profile_reset(ctx._h))


def gp_profile_collect(ctx):
    """gp_profile_count + gp_profile_get for every recorded launch, summed per kernel name:
    {name: dict(launches, ms, flops, bytes)}."""
    lib = load()
    n = C.c_int64()
    ctx.check(lib.gp_profile_count(ctx._h, C.byref(n)))
    out = {}
    name, ms, fl, by = C.c_char_p(), C.c_float(), C.c_double(), C.c_double()
    for i in range(n.value):
        ctx.check(lib.gp_profile_get(ctx._h, C.c_int64(i), C.byref(name), C.byref(ms), C.byref(fl), C.byref(by)))
        d = out.setdefault(name.value.decode(), dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
        d["launches"] += 1
        d["ms"] += ms.value
        d["flops"] += fl.value
        d["bytes"] += by.value
    return out


def _empty(ctx, n, dtype):
    return torch.empty(int(n), dtype=dtype, device=ctx.device)


# ------------------------------------------------------------------ graph
def gp_edges(ctx, pos, graph_ptr, cutoff, max_neighbors=0, cell=None, rep=None):
    """gp_edges_workspace + gp_edges_count + gp_edges_fill.  pos [N,3] f32, graph_ptr [G+1] i32 (device).
    With cell [G,3,3] f32 (device) and rep = (r0, r1, r2): the periodic calls gp_edges_count_pbc / fill_pbc;
    the returned dict then also holds offset [E,3] i32."""
    lib = load()
    n_atoms, n_graphs = pos.shape[0], graph_ptr.shape[0] - 1
    nbytes = C.c_size_t()
    ctx.check(lib.gp_edges_workspace(C.c_int64(n_atoms), C.byref(nbytes)))
    ws = _empty(ctx, max(nbytes.value, 8), torch.uint8)
    n_edges = C.c_int64()
    pbc = cell is not None
    head = (ctx._h, _ptr(pos), _ptr(graph_ptr)) + ((_ptr(cell),) if pbc else ())
    mid = (C.c_int64(n_atoms), C.c_int32(n_graphs), C.c_float(cutoff), C.c_int32(max_neighbors))
    if pbc:
        mid += tuple(C.c_int32(int(r)) for r in rep)
    args = head + mid + (_ptr(ws), C.c_size_t(ws.numel()))
    ctx.check((lib.gp_edges_count_pbc if pbc else lib.gp_edges_count)(*args, C.byref(n_edges)))
    E = n_edges.value
    out = dict(n_atoms=n_atoms, n_edges=E, src=_empty(ctx, E, torch.int32), dst=_empty(ctx, E, torch.int32),
               row_ptr=_empty(ctx, n_atoms + 1, torch.int32), dist=_empty(ctx, E, torch.float32),
               unit=torch.empty((E, 3), dtype=torch.float32, device=ctx.device))
    if pbc:
        out["offset"] = torch.empty((E, 3), dtype=torch.int32, device=ctx.device)
        ctx.check(lib.gp_edges_fill_pbc(*args, C.c_int64(E), _ptr(out["src"]), _ptr(out["dst"]), _ptr(out["offset"]),
                                        _ptr(out["row_ptr"]), _ptr(out["dist"]), _ptr(out["unit"])))
    else:
        ctx.check(lib.gp_edges_fill(*args, C.c_int64(E), _ptr(out["src"]), _ptr(out["dst"]), _ptr(out["row_ptr"]),
                                    _ptr(out["dist"]), _ptr(out["unit"])))
    return out


def gp_triplets(ctx, edges, with_kj=True):
    """gp_triplets_workspace + gp_triplets_count + gp_triplets_fill on an edge dict from gp_edges."""
    lib = load()
    N, E = edges["n_atoms"], edges["n_edges"]
    nbytes = C.c_size_t()
    ctx.check(lib.gp_triplets_workspace(C.c_int64(N), C.c_int64(E), C.byref(nbytes)))
    ws = _empty(ctx, max(nbytes.value, 8), torch.uint8)
    n_trip = C.c_int64()
    pbc = edges.get("offset") is not None     # periodic edge list: image-aware exclusion of k = i
    args = (ctx._h, _ptr(edges["src"]), _ptr(edges["dst"])) + ((_ptr(edges["offset"]),) if pbc else ()) + (
        _ptr(edges["row_ptr"]), C.c_int64(N), C.c_int64(E), _ptr(ws), C.c_size_t(ws.numel()))
    ctx.check((lib.gp_triplets_count_pbc if pbc else lib.gp_triplets_count)(*args, C.byref(n_trip)))
    T = n_trip.value
    out = dict(n_edges=E, n_triplets=T, idx_kj=_empty(ctx, T, torch.int32), idx_ji=_empty(ctx, T, torch.int32),
               seg_ptr_ji=_empty(ctx, E + 1, torch.int32))
    if with_kj:
        out.update(perm_kj=_empty(ctx, T, torch.int32), idx_ji_kj=_empty(ctx, T, torch.int32),
                   seg_ptr_kj=_empty(ctx, E + 1, torch.int32))
    ctx.check((lib.gp_triplets_fill_pbc if pbc else lib.gp_triplets_fill)(*args, C.c_int64(T), _ptr(out["idx_kj"]), _ptr(out["idx_ji"]),
                                   _ptr(out["seg_ptr_ji"]), _ptr(out.get("perm_kj")), _ptr(out.get("idx_ji_kj")),
                                   _ptr(out.get("seg_ptr_kj"))))
    if with_kj and E > 0:
        # lists by centre atom (optional members of gp_graph)
        out_ptr, out_list = gp_edges_by_source(ctx, edges)
        md = C.c_int32()
        ctx.check(lib.gp_csr_max_degree(ctx._h, _ptr(edges["row_ptr"]), C.c_int64(N), _ptr(ws), C.c_size_t(ws.numel()),
                                        C.byref(md)))
        mo = C.c_int32()
        ctx.check(lib.gp_csr_max_degree(ctx._h, _ptr(out_ptr), C.c_int64(N), _ptr(ws), C.c_size_t(ws.numel()), C.byref(mo)))
        out.update(n_atoms=N, row_ptr=edges["row_ptr"], out_ptr=out_ptr, out_list=out_list, max_in_degree=md.value,
                   max_out_degree=mo.value, id_swap=gp_reverse_edges(ctx, edges))
    return out


def gp_reverse_edges(ctx, edges):
    """id_swap[E]: id of the opposite edge of every edge, -1 where the list has none."""
    N, E = edges["n_atoms"], edges["n_edges"]
    out = torch.empty(E, dtype=torch.int32, device=ctx.device)
    ctx.check(load().gp_reverse_edges(ctx._h, _ptr(edges["src"]), _ptr(edges["dst"]), _ptr(edges.get("offset")),
                                      _ptr(edges["row_ptr"]), C.c_int64(N), C.c_int64(E), _ptr(out)))
    return out


def gp_edges_by_source(ctx, edges):
    """out_ptr[N+1], out_list[E]: ids of the edges grouped by source atom."""
    lib = load()
    N, E = edges["n_atoms"], edges["n_edges"]
    nb = C.c_size_t()
    ctx.check(lib.gp_edges_by_source_workspace(C.c_int64(N), C.c_int64(E), C.byref(nb)))
    ws = torch.empty(max(nb.value, 8), dtype=torch.uint8, device=ctx.device)
    out_ptr = torch.empty(N + 1, dtype=torch.int32, device=ctx.device)
    out_list = torch.empty(E, dtype=torch.int32, device=ctx.device)
    ctx.check(lib.gp_edges_by_source(ctx._h, _ptr(edges["src"]), C.c_int64(N), C.c_int64(E), _ptr(ws),
                                     C.c_size_t(ws.numel()), _ptr(out_ptr), _ptr(out_list)))
    return out_ptr, out_list


def gp_edges_by_source_static(ctx, src, n_atoms, out_ptr, out_list):
    """The allocation-free variant: inputs and outputs only (all given by the caller), scratch inside the library."""
    ctx.check(load().gp_edges_by_source_static(ctx._h, _ptr(src), C.c_int64(n_atoms), C.c_int64(src.shape[0]),
                                               _ptr(out_ptr), _ptr(out_list)))
    return out_ptr, out_list


def build_graph(ctx, pos, graph_ptr, cutoff, max_neighbors=0, cell=None, rep=None):
    """Edges and triplets for device tensors pos / graph_ptr (periodic with cell [G,3,3] and rep); returns
    (edges dict, triplets dict)."""
    e = gp_edges(ctx, pos, graph_ptr, cutoff, max_neighbors, cell, rep)
    return e, gp_triplets(ctx, e)


# ------------------------------------------------------------------ basis
def gp_basis_forward(ctx, dims, edges, trip, want_sbf=False):
    lib = load()
    E, T = edges["n_edges"], trip["n_triplets"]
    S, R = dims.num_spherical, dims.num_radial
    out = dict(rbf=torch.empty((E, R), dtype=torch.float32, device=ctx.device),
               cos_alpha=_empty(ctx, T, torch.float32))
    if dims.variant == "D":
        out["rad"] = torch.empty((E, S * R), dtype=torch.float32, device=ctx.device)
    if "perm_kj" in trip:
        out["cos_alpha_kj"] = _empty(ctx, T, torch.float32)
    if want_sbf:
        out["sbf"] = torch.empty((T, S * R), dtype=torch.float32, device=ctx.device)
    d = Dims(dims)
    ctx.check(lib.gp_basis_forward(ctx._h, C.byref(d), _ptr(edges["dist"]), _ptr(edges["unit"]), _ptr(trip["idx_kj"]),
                                   _ptr(trip["idx_ji"]), _ptr(trip.get("perm_kj")), C.c_int64(E), C.c_int64(T),
                                   _ptr(out["rbf"]), _ptr(out.get("rad")), _ptr(out["cos_alpha"]),
                                   _ptr(out.get("cos_alpha_kj")), _ptr(out.get("sbf"))))
    return out


# ------------------------------------------------------------------ block
def gp_block_workspace(dims, n_edges, n_triplets, n_atoms=0):
    lib = load()
    d = Dims(dims)
    a, b = C.c_size_t(), C.c_size_t()
    rc = lib.gp_block_workspace(C.byref(d), C.c_int64(n_atoms), C.c_int64(n_edges), C.c_int64(n_triplets), C.byref(a), C.byref(b))
    if rc != 0:
        raise GpError(rc, "gp_block_workspace")
    return a.value, b.value


def gp_block_forward_D(ctx, dims, w, trip, basis, m_in, m_out, saved, scratch):
    lib = load()
    d, g, b, ws = Dims(dims), Graph(trip), Basis(basis), _weights_D(dims, w)
    ctx.check(lib.gp_block_forward_D(ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), _ptr(m_in), _ptr(m_out),
                                     _ptr(saved), C.c_size_t(saved.numel()), _ptr(scratch), C.c_size_t(scratch.numel())))
    return m_out


def gp_block_backward_D(ctx, dims, w, trip, basis, m_in, saved, grad_m_out, grad_m_in, grad_w, scratch):
    lib = load()
    d, g, b = Dims(dims), Graph(trip), Basis(basis)
    ws, gws = _weights_D(dims, w), _weights_D(dims, grad_w)
    ctx.check(lib.gp_block_backward_D(ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), _ptr(m_in), _ptr(saved),
                                      C.c_size_t(saved.numel()), _ptr(grad_m_out), _ptr(grad_m_in), C.byref(gws),
                                      _ptr(scratch), C.c_size_t(scratch.numel())))
    return grad_m_in, grad_w


def gp_block_backward_D_basis(ctx, dims, w, trip, basis, m_in, saved, grad_m_out, grad_m_in, grad_w, scratch,
                              grad_rbf=None, grad_rad=None, grad_cos_kj=None, accumulate=False):
    """gp_block_backward_D plus the gradients with respect to the basis (written into the given tensors)."""
    lib = load()
    d, g, b = Dims(dims), Graph(trip), Basis(basis)
    ws, gws = _weights_D(dims, w), _weights_D(dims, grad_w)
    ctx.check(lib.gp_block_backward_D_basis(ctx._h, C.byref(d), C.byref(ws), C.byref(g), C.byref(b), _ptr(m_in), _ptr(saved),
                                            C.c_size_t(saved.numel()), _ptr(grad_m_out), _ptr(grad_m_in), C.byref(gws),
                                            _ptr(grad_rbf), _ptr(grad_rad), _ptr(grad_cos_kj), C.c_int32(1 if accumulate else 0),
                                            _ptr(scratch), C.c_size_t(scratch.numel())))
    return grad_m_in, grad_w


# ------------------------------------------------------------------ core kernels on their own
def gp_triplet_aggregate_fwd(ctx, trip, x, s, a=None):
    lib = load()
    g = Graph(trip)
    if a is None:
        a = torch.empty_like(x)
    ctx.check(lib.gp_triplet_aggregate_fwd(ctx._h, C.byref(g), C.c_int32(x.shape[1]), _ptr(x), _ptr(s), _ptr(a)))
    return a


def gp_triplet_aggregate_bwd(ctx, trip, x, s, grad_a):
    lib = load()
    g = Graph(trip)
    gx, gs = torch.empty_like(x), torch.empty_like(s)
    ctx.check(lib.gp_triplet_aggregate_bwd(ctx._h, C.byref(g), _ptr(trip["perm_kj"]), C.c_int32(x.shape[1]), _ptr(x),
                                           _ptr(s), _ptr(grad_a), _ptr(gx), _ptr(gs)))
    return gx, gs


TRIPLET_STREAM, TRIPLET_PER_EDGE, TRIPLET_PER_ATOM, TRIPLET_PER_ATOM_TWO_KERNELS = 0, 1, 2, 3


def gp_triplet_workspace(ctx, trip, width):
    """Scratch tensor for the per-centre-atom forms of the stand-alone triplet kernels."""
    g = Graph(trip)
    nb = C.c_size_t()
    rc = load().gp_triplet_workspace(C.byref(g), C.c_int32(width), C.byref(nb))
    if rc != 0:
        raise GpError(rc, "gp_triplet_workspace")
    return torch.empty(max(nb.value, 8), dtype=torch.uint8, device=ctx.device)


def gp_triplet_hadamard_fwd(ctx, trip, form, S, cos_alpha, x, Qt, W2, want_Bacc=True):
    """a [E,F], Bacc [E,B,F] (or None).  Qt [S*B, E], W2 [B, F]."""
    g = Graph(trip)
    B_, F = W2.shape
    a = torch.empty_like(x)
    Bacc = torch.empty((x.shape[0], B_, F), dtype=torch.float32, device=ctx.device) if want_Bacc else None
    ctx.check(load().gp_triplet_hadamard_fwd(ctx._h, C.byref(g), C.c_int32(form), C.c_int32(S), C.c_int32(B_), C.c_int32(F),
                                             _ptr(cos_alpha), _ptr(x), _ptr(Qt), _ptr(W2), _ptr(a), _ptr(Bacc)))
    return a, Bacc


def gp_triplet_hadamard_bwd(ctx, trip, form, S, cos_alpha_kj, x, Qt, W2, grad_a, ws=None):
    """grad_x [E,F], grad_Q [E,S,B], grad_W2 [B,F] (per-atom form only, else None)."""
    g = Graph(trip)
    B_, F = W2.shape
    gx = torch.empty_like(x)
    gQ = torch.empty((x.shape[0], S, B_), dtype=torch.float32, device=ctx.device)
    gW2 = torch.empty_like(W2) if form == TRIPLET_PER_ATOM else None
    ctx.check(load().gp_triplet_hadamard_bwd(ctx._h, C.byref(g), C.c_int32(form), C.c_int32(S), C.c_int32(B_), C.c_int32(F),
                                             _ptr(cos_alpha_kj), _ptr(x), _ptr(Qt), _ptr(W2), _ptr(grad_a), _ptr(gx), _ptr(gQ),
                                             _ptr(gW2), _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0)))
    return gx, gQ, gW2


def gp_triplet_bilinear_fwd(ctx, trip, form, S, Cc, cos_alpha, x, Radt, ws=None):
    """A [E, C, F] fp32.  Radt [S*C, E]."""
    g = Graph(trip)
    A = torch.empty((x.shape[0], Cc, x.shape[1]), dtype=torch.float32, device=ctx.device)
    ctx.check(load().gp_triplet_bilinear_fwd(ctx._h, C.byref(g), C.c_int32(form), C.c_int32(S), C.c_int32(Cc), C.c_int32(x.shape[1]),
                                             _ptr(cos_alpha), _ptr(x), _ptr(Radt), _ptr(A), _ptr(ws),
                                             C.c_size_t(ws.numel() if ws is not None else 0)))
    return A


def gp_triplet_bilinear_bwd_H(ctx, trip, form, S, cos_alpha_kj, dz, ws=None):
    """H [E, S, O]."""
    g = Graph(trip)
    H = torch.empty((dz.shape[0], S, dz.shape[1]), dtype=torch.float32, device=ctx.device)
    ctx.check(load().gp_triplet_bilinear_bwd_H(ctx._h, C.byref(g), C.c_int32(form), C.c_int32(S), C.c_int32(dz.shape[1]),
                                               _ptr(cos_alpha_kj), _ptr(dz), _ptr(H), _ptr(ws),
                                               C.c_size_t(ws.numel() if ws is not None else 0)))
    return H


def gp_triplet_bilinear_grad_cos(ctx, trip, form, S, cos_alpha_kj, U, dz, grad_cos_kj=None, ws=None):
    """grad_cos_kj [T] (kj-major); added to the given tensor, else a new one is written."""
    g = Graph(trip)
    acc = grad_cos_kj is not None
    out = grad_cos_kj if acc else torch.empty(trip["n_triplets"], dtype=torch.float32, device=ctx.device)
    ctx.check(load().gp_triplet_bilinear_grad_cos(ctx._h, C.byref(g), C.c_int32(form), C.c_int32(S), C.c_int32(dz.shape[1]),
                                                  _ptr(cos_alpha_kj), _ptr(U), _ptr(dz), C.c_int32(1 if acc else 0), _ptr(out),
                                                  _ptr(ws), C.c_size_t(ws.numel() if ws is not None else 0)))
    return out


def gp_linear_forward(ctx, x, W, b=None, act=0, bf16=False):
    lib = load()
    out = torch.empty((x.shape[0], W.shape[1]), dtype=torch.float32, device=ctx.device)
    fn = lib.gp_linear_forward_bf16 if bf16 else lib.gp_linear_forward
    ctx.check(fn(ctx._h, _ptr(x), _ptr(W), _ptr(b), C.c_int64(x.shape[0]), C.c_int32(W.shape[0]),
                                    C.c_int32(W.shape[1]), C.c_int32(act), _ptr(out)))
    return out
