"""Build the oracle's state for a workload description.  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

from .gear_oracle import GearOracle, Precision


def oracle_for(wl, dfv_seed=None) -> GearOracle:
    """Oracle with lazily materialised tables from the counter-based initialiser, in the workload's
    storage types (wl: any object with the fields of gear_inputs.GearWorkload)."""
    prec = Precision(emb=wl.emb_dtype, dfv=wl.dfv_dtype, mlp=wl.mlp_dtype, master="f32")
    return GearOracle.from_seed(wl.seed, wl.n_users, wl.n_urls, wl.n_images, wl.emb_dim, wl.dfv_dim,
                                wl.layers, wl.M, prec, emb_std=wl.emb_std, dfv_std=wl.dfv_std, dfv_seed=dfv_seed)
