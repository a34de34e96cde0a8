"""Seeded page-view batches (Section 1, Table 1: user id, URL, several image ids).

A batch is a CSR list of image ids per page view plus one user id, one URL
bucket and one click label per view.  Ids follow a Zipf law over ranks, and a
fixed bijection spreads the ranks over the id space so that hot rows are not
neighbours in memory.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

from .configs import GearWorkload


@dataclass
class PageViewBatch:
    user_id: np.ndarray   # [B]     int32
    url_id: np.ndarray    # [B]     int32
    img_off: np.ndarray   # [B+1]   int32, img_off[0] = 0, img_off[B] = nnz
    img_id: np.ndarray    # [nnz]   int32, flat CSR order (view, then slot)
    label: np.ndarray     # [B]     float32 in {0, 1}

    @property
    def B(self) -> int:
        return int(self.user_id.shape[0])

    @property
    def nnz(self) -> int:
        return int(self.img_id.shape[0])


class ZipfIds:
    """ids with p(rank r) proportional to r^-s on ranks 1..N, s = 0 is uniform.

    Ranks are drawn by inverse CDF in fp64 and mapped to ids by
    id = (a * (r - 1) + c) mod N with gcd(a, N) = 1.
    """

    def __init__(self, n: int, s: float, salt: int):
        self.n = int(n)
        self.s = float(s)
        a = (2654435761 + 2 * salt * 40503) % self.n
        if a < 2:
            a = 1
        while math.gcd(a, self.n) != 1:
            a += 1
        self.a = a if self.n > 1 else 1
        self.c = (0x9E3779B1 * (salt + 1)) % self.n
        self._cdf = None
        if self.s > 0.0:
            w = np.arange(1, self.n + 1, dtype=np.float64)
            np.power(w, -self.s, out=w)
            np.cumsum(w, out=w)
            w /= w[-1]
            self._cdf = w

    def ranks(self, rng: np.random.Generator, count: int) -> np.ndarray:
        """0-based ranks."""
        if self._cdf is None:
            return rng.integers(0, self.n, size=count, dtype=np.int64)
        u = rng.random(count)
        r = np.searchsorted(self._cdf, u, side="right")
        return np.minimum(r, self.n - 1).astype(np.int64)

    def rank_to_id(self, r: np.ndarray) -> np.ndarray:
        # a < 2^32 and r < 2^26 keep the product inside int64
        return ((r * self.a + self.c) % self.n).astype(np.int32)

    def sample(self, rng: np.random.Generator, count: int) -> np.ndarray:
        return self.rank_to_id(self.ranks(rng, count))


class PageViewSource:
    """Stream of batches for one workload; batch(step) is a pure function of (seed, step)."""

    def __init__(self, wl: GearWorkload):
        self.wl = wl
        self.users = ZipfIds(wl.n_users, wl.zipf_user, salt=1)
        self.urls = ZipfIds(wl.n_urls, wl.zipf_url, salt=2)
        self.images = ZipfIds(wl.n_images, wl.zipf_image, salt=3)

    def batch(self, step: int, batch: int | None = None) -> PageViewBatch:
        wl = self.wl
        B = wl.batch if batch is None else int(batch)
        rng = np.random.Generator(np.random.Philox(key=[wl.seed, step]))
        n_img = rng.integers(1, wl.max_images + 1, size=B, dtype=np.int64)
        img_off = np.zeros(B + 1, dtype=np.int64)
        np.cumsum(n_img, out=img_off[1:])
        nnz = int(img_off[-1])
        user_id = self.users.sample(rng, B)
        url_id = self.urls.sample(rng, B)
        if wl.image_pattern == "epoch":
            # view b of step t shows image number (t * B + b) mod N of a fixed shuffle of the image set
            assert wl.max_images == 1
            img_id = self.images.rank_to_id((np.int64(step) * B + np.arange(B, dtype=np.int64)) % wl.n_images)
        else:
            img_id = self.images.sample(rng, nnz)
        return PageViewBatch(
            user_id=user_id,
            url_id=url_id,
            img_off=img_off.astype(np.int32),
            img_id=img_id,
            label=(rng.random(B) < wl.label_p).astype(np.float32),
        )


def batch_from_lists(user_id, url_id, images_per_view, label) -> PageViewBatch:
    """Build a batch from explicit Python lists (worked examples, edge cases)."""
    B = len(user_id)
    off = np.zeros(B + 1, dtype=np.int32)
    flat = []
    for b, imgs in enumerate(images_per_view):
        flat.extend(int(i) for i in imgs)
        off[b + 1] = len(flat)
    return PageViewBatch(
        user_id=np.asarray(user_id, dtype=np.int32).reshape(B),
        url_id=np.asarray(url_id, dtype=np.int32).reshape(B),
        img_off=off,
        img_id=np.asarray(flat, dtype=np.int32).reshape(len(flat)),
        label=np.asarray(label, dtype=np.float32).reshape(B),
    )
