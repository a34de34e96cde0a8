"""Workload shapes for the Gear Training sparse-part step.

Each workload stands in for the paper's advertisement page-view logs
(Section 1, Table 1: a page view is a user id, a URL and several image ids;
Section 5: few images shared by many page views).  The logs themselves are
proprietary, so every field below is synthetic and seeded.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class GearWorkload:
    name: str
    batch: int                 # page views per step
    steps: int                 # steps of a full run
    n_users: int
    n_urls: int
    n_images: int
    emb_dim: int               # width of a user / URL embedding row
    dfv_dim: int               # width of a Dense Feature Vector
    emb_dtype: str             # "f32" | "bf16"
    dfv_dtype: str             # "f32" | "bf16"
    mlp_dtype: str             # "f32" | "bf16"  (operand type of the MLP contractions)
    max_images: int            # images per view ~ Uniform{1..max_images}
    zipf_user: float           # exponent s of p(r) ~ r^-s ; 0 = uniform
    zipf_url: float
    zipf_image: float
    layers: Tuple[int, ...]    # MLP output widths, last is 1 (the logit)
    label_p: float             # labels ~ Bernoulli(label_p)
    M: int                     # gradients averaged per image before an emission
    lr: float
    emb_std: float = 0.01
    dfv_std: float = 1.0
    refresh_every: int = 0     # full DFV refresh period in steps, 0 = never
    seed: int = 20180603
    image_pattern: str = "zipf"  # "zipf": ids drawn per occurrence; "epoch": one image per view, every
                                 # image exactly once per n_images / batch steps (a data set walked in epochs)

    @property
    def in_features(self) -> int:
        return 2 * self.emb_dim + self.dfv_dim

    @property
    def max_nnz(self) -> int:
        return self.batch * self.max_images

    def scaled(self, **kw) -> "GearWorkload":
        return replace(self, **kw)


WORKLOADS = {
    "tiny": GearWorkload(
        name="tiny", batch=512, steps=8, n_users=1_000, n_urls=4_096, n_images=2_000,
        emb_dim=16, dfv_dim=64, emb_dtype="f32", dfv_dtype="f32", mlp_dtype="f32",
        max_images=4, zipf_user=0.0, zipf_url=0.0, zipf_image=0.0,
        layers=(64, 1), label_p=0.05, M=4, lr=0.01),
    "small": GearWorkload(
        name="small", batch=4_096, steps=100, n_users=1_000_000, n_urls=1 << 22,
        n_images=100_000, emb_dim=32, dfv_dim=256, emb_dtype="f32", dfv_dtype="f32",
        mlp_dtype="f32", max_images=8, zipf_user=1.1, zipf_url=1.1, zipf_image=1.1,
        layers=(256, 128, 1), label_p=0.03, M=16, lr=0.01),
    "bf16": GearWorkload(
        name="bf16", batch=16_384, steps=200, n_users=10_000_000, n_urls=1 << 24,
        n_images=1_000_000, emb_dim=32, dfv_dim=512, emb_dtype="bf16", dfv_dtype="bf16",
        mlp_dtype="bf16", max_images=8, zipf_user=1.1, zipf_url=1.1, zipf_image=1.1,
        layers=(512, 256, 1), label_p=0.03, M=32, lr=0.01),
    "hotkey": GearWorkload(
        name="hotkey", batch=16_384, steps=200, n_users=1_000_000, n_urls=1 << 22,
        n_images=10_000, emb_dim=32, dfv_dim=256, emb_dtype="f32", dfv_dtype="f32",
        mlp_dtype="f32", max_images=16, zipf_user=1.1, zipf_url=1.1, zipf_image=1.5,
        layers=(256, 1), label_p=0.03, M=64, lr=0.01),
    "large": GearWorkload(
        name="large", batch=65_536, steps=1_000, n_users=50_000_000, n_urls=1 << 25,
        n_images=4_000_000, emb_dim=64, dfv_dim=1024, emb_dtype="f32", dfv_dtype="bf16",
        mlp_dtype="bf16", max_images=8, zipf_user=1.05, zipf_url=1.05, zipf_image=1.05,
        layers=(1024, 256, 1), label_p=0.03, M=16, lr=0.01, refresh_every=500),
    # The other extreme of image reuse (Section 4.1 trains on a fixed image set split between the two
    # gears): one image per sample, no image twice in an epoch, so a group of M closes only after M
    # epochs and every step touches batch-many cold rows.  50,000 images as in that data set's
    # training split; the sparse ids are few and uniform because that experiment has none.
    "epoch": GearWorkload(
        name="epoch", batch=5_000, steps=100, n_users=100, n_urls=128, n_images=50_000,
        emb_dim=16, dfv_dim=256, emb_dtype="f32", dfv_dtype="f32", mlp_dtype="f32",
        max_images=1, zipf_user=0.0, zipf_url=0.0, zipf_image=0.0,
        layers=(256, 1), label_p=0.1, M=4, lr=0.01, image_pattern="epoch"),
}


def get_workload(name: str) -> GearWorkload:
    return WORKLOADS[name]
