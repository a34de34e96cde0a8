"""A stand-in Dense Part for closing the loop: DFV[i] = Wd raw[i].  TEST INFRASTRUCTURE ONLY.

The paper's Dense Part is a CNN over the raw image; what the method needs from it is an inference
pass whose results fill the cache (Section 3, steps 1-2) and a backward pass that takes the average
of M gradients with respect to an image's DFV (Section 3, step 6).  Eq. 1 splits the gradient of
the loss with respect to the Dense Part's weights into dLoss/dDFV (the Sparse Part's job, averaged
per image) times dDFV/dW (the Dense Part's job).  For a linear map the second factor is the image's
feature vector, so one emission (i, g) moves the weights by  -lr * outer(g, raw[i]).

Plain fp64 numpy; weights and features are fp32 values held exactly.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np

from .rounding import round_f32, round_to


class DenseStandIn:
    def __init__(self, raw: np.ndarray, wd: np.ndarray, dfv_dtype: str):
        self.raw = round_f32(np.asarray(raw, dtype=np.float64))       # [n_images x r]
        self.wd = round_f32(np.asarray(wd, dtype=np.float64))         # [D x r]
        self.dfv_dtype = dfv_dtype
        assert self.raw.shape[1] == self.wd.shape[1]

    def infer(self, image_ids: Sequence[int]) -> np.ndarray:
        """Rows of the cache for the listed images: Wd raw[i], rounded to the cache's type."""
        rows = np.zeros((len(image_ids), self.wd.shape[0]))
        for r, i in enumerate(image_ids):
            if not 0 <= int(i) < self.raw.shape[0]:
                raise ValueError("image id out of range")
            rows[r] = self.wd @ self.raw[int(i)]
        return round_to(rows, self.dfv_dtype)

    def backward(self, ready_ids: Sequence[int], ready_grads: np.ndarray, lr: float) -> None:
        """One SGD step per emission, in ready-list order (Section 3, step 6)."""
        for i in ready_ids:
            if not 0 <= int(i) < self.raw.shape[0]:
                raise ValueError("image id out of range")
        wd = self.wd
        for i, g in zip(ready_ids, np.asarray(ready_grads, dtype=np.float64)):
            wd = wd - lr * np.outer(g, self.raw[int(i)])
        self.wd = round_f32(wd)
