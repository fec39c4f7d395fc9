"""The five benchmark workloads, and one at the widest widths the paper trains, as plain data (shapes and generator
parameters only)."""
from dataclasses import dataclass, field, replace
from typing import Tuple


@dataclass(frozen=True)
class BlockDims:
    """Layer widths of one interaction block.

    variant "D": Hadamard interaction with down/up projection (DimeNet++ shape).
    variant "G": bilinear interaction (GemNet-T shape).
    """
    variant: str
    dtype: str              # "f32" or "bf16" (bf16 GEMM operands, fp32 accumulation)
    emb: int                # edge embedding width
    int_emb: int            # triplet (down-projected) width; emb_trip for variant G
    num_radial: int
    num_spherical: int
    cutoff: float
    envelope_p: int = 5
    basis_emb: int = 0      # variant D: width of the two-step basis projections
    emb_rbf: int = 0        # variant G
    emb_cbf: int = 0        # variant G
    emb_bil: int = 0        # variant G
    n_res_before: int = 1   # variant D
    n_res_after: int = 2    # variant D
    radial_at_target: bool = False   # variant G: radial factor of the triplet basis at the target edge j->i
    symmetric: bool = False          # variant G: couple the two messages on a bond (second up-projection W_up_ac)


@dataclass(frozen=True)
class Workload:
    name: str
    dims: BlockDims
    system: str                       # "cube" | "slab" | "box"
    system_args: Tuple = field(default_factory=tuple)
    max_neighbors: int = 0            # 0 = no cap
    n_blocks: int = 1
    head_hidden: int = 0              # >0: per-atom energy head (force workload)


CONFIGS = {
    # 24 atoms uniform in a 6 A cube, min pair distance 0.9 A
    "cfg1": Workload(
        name="cfg1",
        dims=BlockDims(variant="D", dtype="f32", emb=32, int_emb=16, basis_emb=4,
                       num_radial=6, num_spherical=7, cutoff=5.0),
        system="cube", system_args=(24, 6.0, 0.9), max_neighbors=0, n_blocks=1),
    # 16 graphs x (64 slab + 16 adsorbate) atoms
    "cfg2": Workload(
        name="cfg2",
        dims=BlockDims(variant="D", dtype="f32", emb=256, int_emb=64, basis_emb=8,
                       num_radial=6, num_spherical=7, cutoff=6.0),
        system="slab", system_args=(16, 4, 4, 4, 16), max_neighbors=50, n_blocks=4),
    # 8 graphs x (160 slab + 40 adsorbate) atoms
    "cfg3": Workload(
        name="cfg3",
        dims=BlockDims(variant="G", dtype="bf16", emb=512, int_emb=64, emb_rbf=16,
                       emb_cbf=16, emb_bil=64, num_radial=128, num_spherical=7, cutoff=6.0),
        system="slab", system_args=(8, 8, 5, 4, 40), max_neighbors=50, n_blocks=1),
    # 1000 atoms at 0.08 atoms/A^3
    "cfg4": Workload(
        name="cfg4",
        dims=BlockDims(variant="G", dtype="bf16", emb=1024, int_emb=128, emb_rbf=16,
                       emb_cbf=16, emb_bil=64, num_radial=128, num_spherical=7, cutoff=12.0),
        system="box", system_args=(1000, 0.08, 0.9), max_neighbors=0, n_blocks=1),
    "cfg5": Workload(
        name="cfg5",
        dims=BlockDims(variant="G", dtype="bf16", emb=1024, int_emb=128, emb_rbf=16,
                       emb_cbf=16, emb_bil=64, num_radial=128, num_spherical=7, cutoff=12.0),
        system="box", system_args=(1000, 0.08, 0.9), max_neighbors=0, n_blocks=3,
        head_hidden=256),
    # DimeNet++-XL widths (Sec. 4.1: hidden 2048, triplet width 256; the paper's 4 blocks) on the config-2 structures
    "xl": Workload(
        name="xl",
        dims=BlockDims(variant="D", dtype="f32", emb=2048, int_emb=256, basis_emb=8,
                       num_radial=6, num_spherical=7, cutoff=6.0),
        system="slab", system_args=(16, 4, 4, 4, 16), max_neighbors=50, n_blocks=4),
}


def get_workload(name: str, **dim_overrides) -> Workload:
    w = CONFIGS[name]
    if dim_overrides:
        w = replace(w, dims=replace(w.dims, **dim_overrides))
    return w
