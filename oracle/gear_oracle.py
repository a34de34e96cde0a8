"""One Gear Training sparse-part step, written out plainly.  TEST INFRASTRUCTURE ONLY.

What is computed, and where the paper says so:

  * A page view is a user id, a URL and several image ids (Section 1, Table 1).
  * The Dense Part's output for an image, its Dense Feature Vector (DFV), is
    not recomputed: it is fetched by image id from a cache that is overwritten
    from time to time (Section 1, second point; Section 3, steps 1-3).
  * With the DFVs in hand the Fastgear Worker runs the Sparse Part forward to
    the loss, back-propagates through the Sparse Part only, applies the Sparse
    Part's gradients, and keeps the gradient of the loss with respect to each
    DFV (Section 3, step 4; Eq. 1, left factor).
  * Each (image id, dLoss/dDFV) pair is handed to the gradient store (Section 3,
    step 5).  Every gradient of an image is stored; when M of them have
    arrived they are averaged and that average is what the Dense Part would
    back-propagate (Section 1, third point; Section 3, step 6).

The paper's model figure is lost, so the Sparse Part used here is the one the
workloads name: x = [user embedding | URL embedding | mean of the view's DFVs],
an MLP with ReLU hidden layers and one logit, sigmoid cross-entropy averaged
over the batch, plain SGD.

Arithmetic is fp64.  `round_to` is applied only where a workload *stores* a
value in a narrower type (tables, bf16 MLP operands and deltas); see `Precision`.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import philox_normal
from .rounding import round_f32, round_to

STREAM_USER = 1
STREAM_URL = 2
STREAM_DFV = 3
STREAM_MLP = 16      # + layer index


@dataclass(frozen=True)
class Precision:
    """Storage types.  "f64" everywhere turns every rounding off (pure mathematics)."""
    emb: str = "f32"     # user / URL embedding rows
    dfv: str = "f32"     # cached DFVs
    mlp: str = "f32"     # operand type of the MLP contractions; "bf16" rounds x, W, h, delta
    master: str = "f32"  # MLP master parameters

    @staticmethod
    def exact() -> "Precision":
        return Precision("f64", "f64", "f64", "f64")


class RowStore:
    """A table of rows keyed by integer id, materialised on first use.

    Either backed by an explicit dense array or by `filler(ids) -> rows`
    (the counter-based initialiser), so that a 50M-row table costs only the
    rows a run touches.  Rows are held as fp64 copies of the stored values.
    """

    def __init__(self, n_rows: int, dim: int, dtype: str,
                 dense: Optional[np.ndarray] = None,
                 filler: Optional[Callable[[np.ndarray], np.ndarray]] = None):
        self.n_rows, self.dim, self.dtype = int(n_rows), int(dim), dtype
        self._rows: Dict[int, np.ndarray] = {}
        self._dense = None
        self._filler = filler
        if dense is not None:
            dense = np.asarray(dense, dtype=np.float64).reshape(self.n_rows, self.dim)
            self._dense = round_to(dense, dtype).copy()
        elif filler is None:
            self._dense = np.zeros((self.n_rows, self.dim))

    def prefetch(self, ids: Sequence[int]) -> None:
        if self._dense is not None:
            return
        need = sorted({int(i) for i in ids} - self._rows.keys())
        if need:
            block = round_to(np.asarray(self._filler(np.asarray(need)), dtype=np.float64), self.dtype)
            for i, r in zip(need, block):
                self._rows[i] = r.copy()

    def row(self, i: int) -> np.ndarray:
        i = int(i)
        if not 0 <= i < self.n_rows:
            raise IndexError(f"row {i} outside [0, {self.n_rows})")
        if self._dense is not None:
            return self._dense[i]
        if i not in self._rows:
            self.prefetch([i])
        return self._rows[i]

    def set_row(self, i: int, value: np.ndarray) -> None:
        v = round_to(np.asarray(value, dtype=np.float64).reshape(self.dim), self.dtype)
        if self._dense is not None:
            self._dense[int(i)] = v
        else:
            self._rows[int(i)] = v.copy()

    def rows(self, ids: Sequence[int]) -> np.ndarray:
        self.prefetch(ids)
        return np.stack([self.row(i) for i in ids]) if len(ids) else np.zeros((0, self.dim))


@dataclass
class AdamState:
    """Constants, step number and moments (keyed by parameter array / table row) of Adam."""
    beta1: float
    beta2: float
    eps: float
    t: int = 0
    moments: Dict = field(default_factory=dict)


@dataclass
class StepResult:
    loss: float
    ready_ids: np.ndarray          # [n_ready] int32, ascending image id, then emission order
    ready_grads: np.ndarray        # [n_ready x D] averaged dLoss/dDFV
    x: np.ndarray                  # [B x F] MLP input
    logits: np.ndarray             # [B]
    dx: np.ndarray                 # [B x F] dLoss/dx
    grads: List[Tuple[np.ndarray, np.ndarray]]       # (dW_l, db_l)
    occ_grads: np.ndarray          # [nnz x D] dLoss/dDFV per occurrence, flat CSR order
    kink_margin: np.ndarray        # [B x hidden layers] min over the layer's units of |a| / max|a|
    dx_own: Optional[np.ndarray] = None   # dLoss/dx with every ReLU decided by this oracle's own arithmetic (= dx unless relu_choice changed a unit)
    near_units: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))     # [B] hidden units within kink_tol of the kink
    active_units: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))   # [B] active units of the view's sparsest hidden layer
    chosen_units: int = 0          # near-kink units whose branch was taken from relu_choice against the own decision
    chosen_per_view: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))   # [B] the same, per view
    refused_units: int = 0         # units where relu_choice disagreed but the pre-activation is not near the kink (own decision kept)
    emb_term_scale: Dict = field(default_factory=dict)   # ("user"|"url", id) -> largest |element| of the gradient terms summed into the row
    ready_term_scale: np.ndarray = field(default_factory=lambda: np.zeros(0))   # [n_ready] largest |element| of the M gradients behind each average
    user_unique: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    url_unique: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    img_unique: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))
    img_segoff: np.ndarray = field(default_factory=lambda: np.zeros(1, np.int32))
    img_perm: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))


def stable_groups(keys: np.ndarray):
    """Distinct keys ascending, segment offsets, and the stable grouping permutation.

    perm lists positions so that keys[perm] is ascending and equal keys keep
    their original order; segment s is perm[segoff[s]:segoff[s+1]].
    """
    keys = np.asarray(keys)
    buckets: Dict[int, List[int]] = {}
    for pos, k in enumerate(keys.tolist()):
        buckets.setdefault(k, []).append(pos)
    uniq = sorted(buckets)
    perm: List[int] = []
    segoff = [0]
    for k in uniq:
        perm.extend(buckets[k])
        segoff.append(len(perm))
    return (np.asarray(uniq, dtype=np.int32), np.asarray(segoff, dtype=np.int32),
            np.asarray(perm, dtype=np.int32))


def bce_with_logits(z: np.ndarray, y: np.ndarray) -> np.ndarray:
    """-[y log s(z) + (1-y) log(1-s(z))] in the overflow-free form."""
    return np.maximum(z, 0.0) - z * y + np.log1p(np.exp(-np.abs(z)))


def sigmoid(z: np.ndarray) -> np.ndarray:
    e = np.exp(-np.abs(z))
    return np.where(z >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


class GearOracle:
    """State of one Fastgear Worker plus the Slowgear gradient store, and `step`."""

    def __init__(self, user_emb: RowStore, url_emb: RowStore, dfv: RowStore,
                 mlp: List[Tuple[np.ndarray, np.ndarray]], M: int,
                 precision: Precision = Precision()):
        if M < 1:
            raise ValueError("M must be >= 1")
        self.user_emb, self.url_emb, self.dfv = user_emb, url_emb, dfv
        self.prec = precision
        self.mlp = [(round_to(np.array(W, dtype=np.float64), precision.master),
                     round_to(np.array(b, dtype=np.float64).reshape(-1), precision.master))
                    for W, b in mlp]
        self.M = int(M)
        self.d = user_emb.dim
        self.D = dfv.dim
        self.F = 2 * self.d + self.D
        assert url_emb.dim == self.d and self.mlp[0][0].shape[1] == self.F
        assert self.mlp[-1][0].shape[0] == 1
        # Section 1, third point: every gradient of an image is kept until M have arrived.
        self.store: Dict[int, List[np.ndarray]] = {}
        self.counts: Dict[int, int] = {}
        self.stamps: Dict[int, int] = {}     # image id -> time its cached DFV was last written
        self.stamp0 = 0                      # ... for rows never stamped
        self.adam: Optional[AdamState] = None   # None = plain SGD

    # ---- construction from the counter-based initialiser ------------------------------------
    @staticmethod
    def from_seed(seed: int, n_users: int, n_urls: int, n_images: int, emb_dim: int,
                  dfv_dim: int, layers: Sequence[int], M: int, precision: Precision,
                  emb_std: float = 0.01, dfv_std: float = 1.0,
                  dfv_seed: Optional[int] = None) -> "GearOracle":
        def filler(stream, dim, std, sd=seed):
            return lambda ids: philox_normal.normal_rows(sd, stream, ids, dim, std)
        user = RowStore(n_users, emb_dim, precision.emb, filler=filler(STREAM_USER, emb_dim, emb_std))
        url = RowStore(n_urls, emb_dim, precision.emb, filler=filler(STREAM_URL, emb_dim, emb_std))
        dfv = RowStore(n_images, dfv_dim, precision.dfv,
                       filler=filler(STREAM_DFV, dfv_dim, dfv_std, seed if dfv_seed is None else dfv_seed))
        mlp = []
        fan_in = 2 * emb_dim + dfv_dim
        for l, width in enumerate(layers):
            W = philox_normal.normal_rows(seed, STREAM_MLP + l, np.arange(width), fan_in,
                                          float(np.sqrt(2.0 / fan_in)))
            mlp.append((W.astype(np.float64), np.zeros(width)))
            fan_in = width
        return GearOracle(user, url, dfv, mlp, M, precision)

    # ---- cache refresh (Section 1, second point: cached results are overwritten) -------------
    def refresh_dfv(self, image_ids: Sequence[int], new_rows: np.ndarray) -> None:
        """Overwrite cached DFVs.  The gradient store and the counters live in another table
        (Section 1, third point) and are not touched."""
        for i, r in zip(image_ids, np.asarray(new_rows, dtype=np.float64)):
            self.dfv.set_row(int(i), r)

    # ---- the update rule ------------------------------------------------------------------------
    def use_adam(self, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
        """Switch from plain SGD to Adam (Section 4.1 names the optimiser, not its constants)."""
        self.adam = AdamState(float(np.float32(beta1)), float(np.float32(beta2)), float(np.float32(eps)))

    def _update(self, key, w: np.ndarray, g: np.ndarray, lr: float) -> np.ndarray:
        """New value of the parameter array `key` (unrounded; the caller rounds to the storage type).
        Adam as in Kingma & Ba, Algorithm 1, with moments kept in fp32; the step number is the
        global one also for table rows, whose moments move only when the row is touched."""
        if self.adam is None:
            return w - lr * g
        a = self.adam
        m, v = a.moments.get(key, (np.zeros_like(w), np.zeros_like(w)))
        m = round_f32(a.beta1 * m + (1.0 - a.beta1) * g)
        v = round_f32(a.beta2 * v + (1.0 - a.beta2) * g * g)
        a.moments[key] = (m, v)
        step = lr / (1.0 - a.beta1 ** a.t)
        return w - step * m / (np.sqrt(v) / np.sqrt(1.0 - a.beta2 ** a.t) + a.eps)

    # ---- expiry of cached inference results (Section 1, second point; Section 3; Table 2) ------
    def expired(self, image_ids: Sequence[int], now: int, expiry: int) -> List[int]:
        """The distinct images among `image_ids` whose cached DFV is at least `expiry` old, ascending.
        A row never stamped has time `self.stamp0`."""
        hits = set()
        for i in image_ids:
            i = int(i)
            if not 0 <= i < self.dfv.n_rows:
                raise ValueError("image id out of range")
            if now - self.stamps.get(i, self.stamp0) >= expiry:
                hits.add(i)
        return sorted(hits)

    def stamp(self, image_ids: Sequence[int], now: int) -> None:
        for i in image_ids:
            self.stamps[int(i)] = int(now)

    def residual(self, image_id: int) -> np.ndarray:
        """Sum of the gradients currently stored for an image (what a running sum would hold)."""
        acc = np.zeros(self.D)
        for g in self.store.get(int(image_id), []):
            acc = acc + g
        return acc

    def residual_term_scale(self, image_id: int) -> float:
        """Largest |element| among the gradients currently stored for an image."""
        return max([float(np.abs(g).max()) for g in self.store.get(int(image_id), [])] or [0.0])

    def receive(self, image_id: int, g: np.ndarray) -> Optional[np.ndarray]:
        """Slowgear bookkeeping for one arriving gradient (Section 1, third point; Section 3,
        step 6): keep it; once M are kept return their average and start collecting afresh."""
        kept = self.store.setdefault(image_id, [])
        kept.append(np.array(g, dtype=np.float64))
        self.counts[image_id] = self.counts.get(image_id, 0) + 1
        if len(kept) < self.M:
            return None
        total = np.zeros_like(kept[0])
        for gk in kept:                                              # arrival order
            total = total + gk
        # size of the largest term of the average: what its rounding error is measured against
        self.last_term_scale = max(float(np.abs(gk).max()) for gk in kept)
        kept.clear()
        return total / self.M

    # ---- one training step -------------------------------------------------------------------
    def _forward_backward(self, x: np.ndarray, y: np.ndarray, relu_choice, kink_tol: float) -> dict:
        """Forward to the loss and backward to dLoss/dx from the current (pre-step) parameters; changes no
        state.  relu_choice (one boolean [B x H_l] array per hidden layer, or None): for units whose
        pre-activation lies within kink_tol * max|a_l| of zero, the branch to take instead of this
        arithmetic's own `a > 0`; everywhere else the own decision stands whatever relu_choice says."""
        B = x.shape[0]
        L = len(self.mlp)
        Wc = [round_to(W, self.prec.mlp) for W, _ in self.mlp]
        h = [x]
        active = [None]                                              # ReLU'(a_l): 1 where a_l > 0
        kink = np.full((B, max(L - 1, 1)), np.inf)
        near_units = np.zeros(B, dtype=np.int64)
        active_units = np.full(B, np.iinfo(np.int64).max, dtype=np.int64)
        chosen = refused = 0
        chosen_per_view = np.zeros(B, dtype=np.int64)
        for l in range(L - 1):
            a = h[l] @ Wc[l].T + self.mlp[l][1]
            scale = np.maximum(np.abs(a).max(axis=1), np.finfo(np.float64).tiny)
            kink[:, l] = np.abs(a).min(axis=1) / scale
            on = a > 0
            near = np.abs(a) < kink_tol * scale[:, None]
            near_units += near.sum(axis=1)
            if relu_choice is not None:
                want = np.asarray(relu_choice[l], dtype=bool)
                differs = want != on
                chosen += int((differs & near).sum())
                chosen_per_view += (differs & near).sum(axis=1)
                refused += int((differs & ~near).sum())
                on = np.where(near, want, on)
            active_units = np.minimum(active_units, on.sum(axis=1))
            active.append(on)
            h.append(round_to(np.where(on, np.maximum(a, 0.0), 0.0), self.prec.mlp))
        z = (h[L - 1] @ Wc[L - 1].T + self.mlp[L - 1][1])[:, 0]
        loss = float(np.sum(bce_with_logits(z, y)) / B) if B else 0.0

        delta = ((sigmoid(z) - y) / max(B, 1)).reshape(B, 1)       # dLoss/dz, mean reduction
        grads: List[Tuple[np.ndarray, np.ndarray]] = [None] * L     # type: ignore
        dx = np.zeros_like(x)
        for l in range(L - 1, -1, -1):
            grads[l] = (delta.T @ h[l], delta.sum(axis=0))
            back = delta @ Wc[l]
            if l > 0:
                # hidden deltas are MLP operands: ReLU mask, then operand rounding
                delta = round_to(np.where(active[l], back, 0.0), self.prec.mlp)
            else:
                # dLoss/dx is never an operand of a contraction again: it stays unrounded
                dx = back
        return dict(z=z, loss=loss, grads=grads, dx=dx, kink=kink, near_units=near_units,
                    active_units=active_units, chosen=chosen, refused=refused, chosen_per_view=chosen_per_view)

    def step(self, batch, lr: float, relu_choice=None, kink_tol: float = 0.0) -> StepResult:
        """One step.  relu_choice / kink_tol: see _forward_backward; with them the step follows the given
        branch at hidden units that are within rounding distance of the ReLU kink (a comparison with
        another arithmetic then does not hinge on which side of zero each landed), and only there."""
        B, d, D, F, M = batch.B, self.d, self.D, self.F, self.M
        user_id, url_id = batch.user_id, batch.url_id
        off, img_id, y = batch.img_off, batch.img_id, batch.label.astype(np.float64)
        if off[0] != 0 or off[B] != len(img_id) or np.any(np.diff(off) < 0):
            raise ValueError("image offsets are not a CSR index")
        self.user_emb.prefetch(user_id)
        self.url_emb.prefetch(url_id)
        self.dfv.prefetch(img_id)

        # 1. Sparse-Part input: embeddings and the mean of the view's cached DFVs.
        x = np.zeros((B, F))
        for b in range(B):
            x[b, :d] = self.user_emb.row(user_id[b])
            x[b, d:2 * d] = self.url_emb.row(url_id[b])
            n_b = off[b + 1] - off[b]
            if n_b > 0:
                pooled = np.zeros(D)
                for j in range(off[b], off[b + 1]):
                    pooled = pooled + self.dfv.row(img_id[j])
                x[b, 2 * d:] = pooled / n_b
        x = round_to(x, self.prec.mlp)

        # 2.-3. Forward to the loss and back-propagation through the Sparse Part only (Section 3, step 4).
        own = self._forward_backward(x, y, None, kink_tol)
        fb = own
        if relu_choice is not None:
            fb = self._forward_backward(x, y, relu_choice, kink_tol)
        z, loss, grads, dx, kink = fb["z"], fb["loss"], fb["grads"], fb["dx"], fb["kink"]

        # 4. Apply the Sparse Part's gradients: plain SGD, or Adam when `self.adam` is set (MLP: every
        #    element; tables: the touched rows only, moments included).
        if self.adam is not None:
            self.adam.t += 1
        emb_term_scale: Dict = {}
        new_mlp = []
        for l, ((W, b), (dW, db)) in enumerate(zip(self.mlp, grads)):
            new_mlp.append((round_to(self._update(("W", l), W, dW, lr), self.prec.master),
                            round_to(self._update(("b", l), b, db, lr), self.prec.master)))
        self.mlp = new_mlp
        for name, table, ids, lo in (("user", self.user_emb, user_id, 0), ("url", self.url_emb, url_id, d)):
            row_grad: Dict[int, np.ndarray] = {}
            for b in range(B):                                       # batch order
                k = int(ids[b])
                row_grad[k] = row_grad.get(k, np.zeros(d)) + dx[b, lo:lo + d]
                emb_term_scale[(name, k)] = max(emb_term_scale.get((name, k), 0.0), float(np.abs(dx[b, lo:lo + d]).max()))
            for k, g in row_grad.items():
                table.set_row(k, self._update((name, k), table.row(k), g, lr))

        # 5. Hand every (image id, dLoss/dDFV) to the gradient store, in flat CSR order.
        occ = np.zeros((len(img_id), D))
        emitted: List[Tuple[int, np.ndarray]] = []
        term_scale: List[float] = []
        for b in range(B):
            n_b = off[b + 1] - off[b]
            for j in range(off[b], off[b + 1]):
                occ[j] = dx[b, 2 * d:] / n_b                         # backward of the mean
                mean = self.receive(int(img_id[j]), occ[j])
                if mean is not None:
                    emitted.append((int(img_id[j]), mean))
                    term_scale.append(self.last_term_scale)

        # 6. Ready list: ascending image id, emissions of one image in the order they happened.
        order = sorted(range(len(emitted)), key=lambda e: (emitted[e][0], e))
        ready_ids = np.asarray([emitted[e][0] for e in order], dtype=np.int32)
        ready_grads = (np.stack([emitted[e][1] for e in order]) if order else np.zeros((0, D)))

        iu, isegoff, iperm = stable_groups(img_id)
        return StepResult(loss=loss, ready_ids=ready_ids, ready_grads=ready_grads, x=x, logits=z,
                          dx=dx, grads=grads, occ_grads=occ, kink_margin=kink, dx_own=own["dx"],
                          near_units=own["near_units"], active_units=own["active_units"],
                          chosen_units=fb["chosen"], refused_units=fb["refused"], chosen_per_view=fb["chosen_per_view"],
                          emb_term_scale=emb_term_scale,
                          user_unique=stable_groups(user_id)[0], url_unique=stable_groups(url_id)[0],
                          img_unique=iu, img_segoff=isegoff, img_perm=iperm,
                          ready_term_scale=np.asarray([term_scale[e] for e in order], dtype=np.float64))
