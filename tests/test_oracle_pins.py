"""Pins for the CPU oracle: things fixed by the paper's statement of the method or by
mathematics, none of which call back into the oracle's own formulas.

  * hand-computed worked examples (tests/golden/worked_examples.json),
  * published known answers of the counter-based generator,
  * a finite-difference check of dLoss/dDFV (Eq. 1, left factor),
  * PyTorch autograd in fp64 as an unrelated differentiator,
  * invariants of the store-all / average-at-M bookkeeping (Section 1, third point).
"""
import copy
import json
import math
import os

import numpy as np
import pytest
import torch

from gear_inputs import PageViewSource, get_workload
from gear_inputs.pageviews import batch_from_lists
from oracle.gear_oracle import (GearOracle, Precision, RowStore, bce_with_logits, sigmoid,
                                stable_groups)
from oracle import philox_normal
from oracle.rounding import round_bf16, round_to


# ------------------------------------------------------------------ helpers
def small_oracle(rng, n_users=7, n_urls=5, n_images=9, d=2, D=3, layers=(4, 3, 1), M=2,
                 prec=Precision.exact()):
    F = 2 * d + D
    mlp, fan = [], F
    for w in layers:
        mlp.append((rng.normal(0, 1.0 / math.sqrt(fan), (w, fan)), rng.normal(0, 0.1, w)))
        fan = w
    return GearOracle(RowStore(n_users, d, prec.emb, dense=rng.normal(0, 1, (n_users, d))),
                      RowStore(n_urls, d, prec.emb, dense=rng.normal(0, 1, (n_urls, d))),
                      RowStore(n_images, D, prec.dfv, dense=rng.normal(0, 1, (n_images, D))),
                      mlp, M, prec)


def random_batch(rng, B, n_users, n_urls, n_images, max_images=3, allow_empty=False):
    views = [list(rng.integers(0, n_images, rng.integers(0 if allow_empty else 1, max_images + 1)))
             for _ in range(B)]
    return batch_from_lists(rng.integers(0, n_users, B), rng.integers(0, n_urls, B), views,
                            rng.integers(0, 2, B))


def oracle_from_example(ex):
    d, D = ex["emb_dim"], ex["dfv_dim"]
    prec = Precision.exact()
    mlp = [(np.array(W), np.array(b)) for W, b in zip(ex["W"], ex["b"])]
    o = GearOracle(RowStore(len(ex["user_emb"]), d, "f64", dense=np.array(ex["user_emb"])),
                   RowStore(len(ex["url_emb"]), d, "f64", dense=np.array(ex["url_emb"])),
                   RowStore(len(ex["dfv"]), D, "f64", dense=np.array(ex["dfv"])), mlp, ex["M"], prec)
    v = ex["views"]
    batch = batch_from_lists([w["user"] for w in v], [w["url"] for w in v],
                             [w["images"] for w in v], [w["label"] for w in v])
    return o, batch


@pytest.fixture(scope="module")
def worked(golden_dir):
    with open(os.path.join(golden_dir, "worked_examples.json")) as f:
        return json.load(f)


# ------------------------------------------------------------------ worked examples
@pytest.mark.parametrize("name", ["one_view", "two_views_dead_units"])
def test_hand_computed_step(worked, name):
    ex = worked[name]
    exp = ex["expect"]
    o, batch = oracle_from_example(ex)
    r = o.step(batch, ex["lr"])
    assert np.array_equal(r.x, np.array(exp["x"]))
    assert np.array_equal(r.logits, np.array(exp["logits"]))
    assert r.loss == pytest.approx(math.log(2.0), rel=1e-15)
    for l in range(2):
        assert np.array_equal(r.grads[l][0], np.array(exp["dW"][l]))
        assert np.array_equal(r.grads[l][1], np.array(exp["db"][l]))
        assert np.array_equal(o.mlp[l][0], np.array(exp["W_after"][l]))
        assert np.array_equal(o.mlp[l][1], np.array(exp["b_after"][l]))
    assert np.array_equal(r.dx, np.array(exp["dx"]))
    for k, v in exp["user_emb_after"].items():
        assert np.array_equal(o.user_emb.row(int(k)), np.array(v))
    for k, v in exp["url_emb_after"].items():
        assert np.array_equal(o.url_emb.row(int(k)), np.array(v))
    assert np.array_equal(r.occ_grads, np.array(exp["occ_grads"]))
    assert r.ready_ids.tolist() == exp["ready_ids"]
    assert np.array_equal(r.ready_grads, np.array(exp["ready_grads"]))
    assert {str(k): v for k, v in o.counts.items()} == exp["counts"]
    for k, v in exp["residual"].items():
        assert np.array_equal(o.residual(int(k)), np.array(v))


@pytest.mark.parametrize("name", ["bf16_hidden_activation_rounds", "bf16_hidden_delta_rounds"])
def test_hand_computed_bf16_roundings_inside_the_network(worked, name):
    """Section 3 step 4 with bf16 operands: hidden activations and hidden deltas are stored in bf16
    before they are operands again.  Both examples are built so that the value to be stored is not a
    bf16 number and so that, with the rounding, the logit is exactly 0 and every gradient is exact."""
    ex = worked[name]
    exp = ex["expect"]
    d, D = ex["emb_dim"], ex["dfv_dim"]
    prec = Precision("f32", "f32", "bf16", "f32")
    mlp = [(np.array(W), np.array(b)) for W, b in zip(ex["W"], ex["b"])]
    o = GearOracle(RowStore(len(ex["user_emb"]), d, prec.emb, dense=np.array(ex["user_emb"])),
                   RowStore(len(ex["url_emb"]), d, prec.emb, dense=np.array(ex["url_emb"])),
                   RowStore(len(ex["dfv"]), D, prec.dfv, dense=np.array(ex["dfv"])), mlp, ex["M"], prec)
    v = ex["views"]
    batch = batch_from_lists([w["user"] for w in v], [w["url"] for w in v], [w["images"] for w in v],
                             [w["label"] for w in v])
    r = o.step(batch, ex["lr"])
    assert np.array_equal(r.x, np.array(exp["x"]))
    assert np.array_equal(r.logits, np.array(exp["logits"]))
    assert r.loss == pytest.approx(math.log(2.0), rel=1e-15)
    for l in range(len(mlp)):
        assert np.array_equal(r.grads[l][0], np.array(exp["dW"][l])), l
        assert np.array_equal(r.grads[l][1], np.array(exp["db"][l])), l
    assert np.array_equal(r.dx, np.array(exp["dx"]))
    assert np.array_equal(r.occ_grads, np.array(exp["occ_grads"]))
    assert r.ready_ids.tolist() == exp["ready_ids"] and np.array_equal(r.ready_grads, np.array(exp["ready_grads"]))
    # the same data without any rounding gives the other value the derivation names: the examples do
    # tell the two apart
    e = GearOracle(RowStore(len(ex["user_emb"]), d, "f64", dense=np.array(ex["user_emb"])),
                   RowStore(len(ex["url_emb"]), d, "f64", dense=np.array(ex["url_emb"])),
                   RowStore(len(ex["dfv"]), D, "f64", dense=np.array(ex["dfv"])), mlp, ex["M"], Precision.exact())
    q = e.step(batch, ex["lr"])
    if "logit_without_rounding" in exp:
        assert q.logits[0] == exp["logit_without_rounding"] and q.loss != r.loss
    if "dx0_without_rounding" in exp:
        assert q.dx[0, 0] == exp["dx0_without_rounding"]


def _bare_store(M):
    z = RowStore(1, 1, "f64")
    return GearOracle(z, z, RowStore(1, 1, "f64"), [(np.zeros((1, 3)), np.zeros(1))], M, Precision.exact())


def test_hand_computed_windows(worked):
    ex = worked["windows_two_steps"]
    o = _bare_store(ex["M"])
    e1 = [m[0] for g in ex["step1"] if (m := o.receive(0, np.array([g]))) is not None]
    assert e1 == ex["expect"]["emit1"] and o.residual(0)[0] == ex["expect"]["residual1"]
    assert o.counts[0] == ex["expect"]["count1"]
    e2 = [m[0] for g in ex["step2"] if (m := o.receive(0, np.array([g]))) is not None]
    assert e2 == ex["expect"]["emit2"] and o.residual(0)[0] == ex["expect"]["residual2"]
    assert o.counts[0] == ex["expect"]["count2"]

    ex = worked["windows_one_step"]
    o = _bare_store(ex["M"])
    e1 = [m[0] for g in ex["step1"] if (m := o.receive(0, np.array([g]))) is not None]
    assert e1 == ex["expect"]["emit1"] and o.residual(0)[0] == ex["expect"]["residual1"]
    assert o.counts[0] == ex["expect"]["count1"]


# ------------------------------------------------------------------ generator and roundings
def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = philox_normal.philox4x32_10(*[np.array([c], dtype=np.uint64) for c in v[:4]], v[4], v[5])
        assert [int(o[0]) for o in out] == v[6:]


def test_initialiser_is_integer_irwin_hall():
    idx = np.arange(1 << 18, dtype=np.uint64) + np.uint64(1 << 33)   # exercises the high counter word
    s = philox_normal.centred_sums(12345, 7, idx)
    assert s.dtype == np.int64 and np.abs(s).max() <= 4 * 65535
    sd = math.sqrt(8 * (65536.0 ** 2 - 1) / 12)
    assert abs(s.mean()) < 5 * sd / math.sqrt(len(s))
    assert abs(s.std() / sd - 1) < 0.01
    v = philox_normal.normal_f32(12345, 7, idx, 0.25)
    assert v.dtype == np.float32 and abs(v.std() / 0.25 - 1) < 0.01
    # kurtosis of a sum of 8 uniforms: 3 - 1.2/8
    assert abs(np.mean((s / sd) ** 4) - (3 - 1.2 / 8)) < 0.05
    # different streams / seeds decorrelate, same arguments repeat
    assert np.array_equal(s, philox_normal.centred_sums(12345, 7, idx))
    assert abs(np.corrcoef(s, philox_normal.centred_sums(12345, 8, idx))[0, 1]) < 0.01
    assert abs(np.corrcoef(s, philox_normal.centred_sums(12346, 7, idx))[0, 1]) < 0.01
    # row/col addressing is the flat index row*dim+col
    rows = philox_normal.normal_rows(5, 2, [3, 10], 4, 1.0)
    flat = philox_normal.normal_f32(5, 2, np.array([12, 13, 14, 15, 40, 41, 42, 43]), 1.0)
    assert np.array_equal(rows.reshape(-1), flat)


def test_round_bf16_exhaustive_and_ties():
    pat = np.arange(1 << 16, dtype=np.uint32)
    vals = (pat << 16).view(np.float32).astype(np.float64)
    finite = np.isfinite(vals)
    assert np.array_equal(round_bf16(vals[finite]), vals[finite])            # fixed points
    # midpoint between consecutive positive bf16 values goes to the even pattern
    p = np.arange(0x0001, 0x7F7F, dtype=np.uint32)
    lo = (p << 16).view(np.float32).astype(np.float64)
    hi = ((p + 1) << 16).view(np.float32).astype(np.float64)
    mid = (lo + hi) / 2
    even = np.where(p % 2 == 0, lo, hi)
    assert np.array_equal(round_bf16(mid), even)
    assert np.array_equal(round_bf16(-mid), -even)
    assert np.array_equal(round_bf16(np.nextafter(mid, np.inf)), hi)
    assert np.array_equal(round_bf16(np.nextafter(mid, -np.inf)), lo)
    assert round_bf16(np.array([3.4e38]))[0] == np.inf and round_bf16(np.array([0.0]))[0] == 0.0


def test_round_bf16_matches_library_cast_on_fp32_inputs():
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 1 << 32, 1 << 20, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    f = f[np.isfinite(f)]
    lib = torch.from_numpy(f.copy()).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_bf16(f.astype(np.float64)), lib)
    assert np.array_equal(round_to(np.array([1 + 2.0 ** -30]), "f32"), np.array([1.0]))


# ------------------------------------------------------------------ loss closed forms
def test_loss_closed_forms():
    assert bce_with_logits(np.array([0.0]), np.array([1.0]))[0] == pytest.approx(math.log(2), rel=1e-15)
    z = np.linspace(-20, 20, 81)
    for y in (0.0, 1.0):
        naive = -(y * np.log(1 / (1 + np.exp(-z))) + (1 - y) * np.log(1 - 1 / (1 + np.exp(-z))))
        assert np.allclose(bce_with_logits(z, np.full_like(z, y)), naive, rtol=1e-7, atol=1e-12)
    big = bce_with_logits(np.array([800.0, -800.0, 800.0, -800.0]), np.array([1.0, 0.0, 0.0, 1.0]))
    assert np.all(np.isfinite(big)) and big[2] == 800.0 and big[3] == 800.0 and big[0] < 1e-300
    assert np.allclose(sigmoid(z), 1 / (1 + np.exp(-z)), rtol=1e-13)
    assert sigmoid(np.array([-800.0]))[0] == 0.0 and sigmoid(np.array([800.0]))[0] == 1.0


def test_zero_weights_give_ln2_and_half_minus_y():
    rng = np.random.default_rng(1)
    o = small_oracle(rng)
    o.mlp = [(np.zeros_like(W), np.zeros_like(b)) for W, b in o.mlp]
    batch = random_batch(rng, 6, 7, 5, 9)
    r = o.step(batch, 0.1)
    assert r.loss == pytest.approx(math.log(2), rel=1e-15)
    assert np.allclose(r.grads[-1][1], np.sum(0.5 - batch.label) / 6)
    assert not r.dx.any()


# ------------------------------------------------------------------ derivatives
def test_dfv_gradient_by_finite_differences():
    """Eq. 1, left factor: the gradients stored for an image in one step sum to dLoss/dDFV[image]."""
    rng = np.random.default_rng(2)
    base = small_oracle(rng, M=1000)
    batch = batch_from_lists([0, 1, 2, 3, 1], [0, 1, 1, 2, 4],
                             [[4, 2], [2, 2, 5], [7], [2, 8, 1], [6, 4]], [1, 0, 0, 1, 0])

    def loss_with(image, col, eps):
        o = copy.deepcopy(base)
        row = o.dfv.row(image).copy()
        row[col] += eps
        o.dfv.set_row(image, row)
        return o.step(batch, 0.0).loss

    ref = copy.deepcopy(base)
    ref.step(batch, 0.0)
    eps = 1e-6
    for image in (7, 2, 4):           # once, four times (twice in one view), twice
        for col in range(3):
            fd = (loss_with(image, col, eps) - loss_with(image, col, -eps)) / (2 * eps)
            assert ref.residual(image)[col] == pytest.approx(fd, rel=2e-6, abs=1e-10)
    assert ref.counts[2] == 4 and ref.counts[7] == 1 and ref.counts[4] == 2


def _torch_step(o, batch, lr):
    """The same model differentiated by autograd (fp64); returns grads of every leaf."""
    t = lambda a: torch.tensor(np.array(a), dtype=torch.float64, requires_grad=True)
    E_u, E_v, Dfv = t(o.user_emb._dense), t(o.url_emb._dense), t(o.dfv._dense)
    Ws = [t(W) for W, _ in o.mlp]
    bs = [t(b) for _, b in o.mlp]
    B = batch.B
    n = torch.tensor(np.diff(batch.img_off), dtype=torch.float64)
    view_of = torch.repeat_interleave(torch.arange(B), torch.tensor(np.diff(batch.img_off)))
    pooled = torch.zeros(B, o.D, dtype=torch.float64).index_add(0, view_of, Dfv[torch.tensor(batch.img_id, dtype=torch.long)])
    pooled = pooled / torch.clamp(n, min=1).unsqueeze(1)
    h = torch.cat([E_u[torch.tensor(batch.user_id, dtype=torch.long)],
                   E_v[torch.tensor(batch.url_id, dtype=torch.long)], pooled], dim=1)
    for l, (W, b) in enumerate(zip(Ws, bs)):
        h = h @ W.T + b
        if l < len(Ws) - 1:
            h = torch.relu(h)
    loss = torch.nn.functional.binary_cross_entropy_with_logits(
        h[:, 0], torch.tensor(batch.label, dtype=torch.float64), reduction="mean")
    loss.backward()
    return loss.item(), E_u.grad.numpy(), E_v.grad.numpy(), Dfv.grad.numpy(), \
        [W.grad.numpy() for W in Ws], [b.grad.numpy() for b in bs]


@pytest.mark.parametrize("seed,allow_empty", [(3, False), (4, True)])
def test_against_autograd(seed, allow_empty):
    rng = np.random.default_rng(seed)
    o = small_oracle(rng, M=10 ** 6)
    batch = random_batch(rng, 17, 7, 5, 9, allow_empty=allow_empty)
    before = copy.deepcopy(o)
    loss, gu, gv, gd, gW, gb = _torch_step(before, batch, 0.3)
    r = o.step(batch, 0.3)
    assert r.loss == pytest.approx(loss, rel=1e-12)
    for l in range(len(gW)):
        assert np.allclose(r.grads[l][0], gW[l], rtol=1e-10, atol=1e-14)
        assert np.allclose(r.grads[l][1], gb[l], rtol=1e-10, atol=1e-14)
        assert np.allclose(o.mlp[l][0], before.mlp[l][0] - 0.3 * gW[l], rtol=1e-12, atol=1e-15)
    assert np.allclose(o.user_emb._dense, before.user_emb._dense - 0.3 * gu, rtol=1e-12, atol=1e-15)
    assert np.allclose(o.url_emb._dense, before.url_emb._dense - 0.3 * gv, rtol=1e-12, atol=1e-15)
    for i in range(9):                       # M is huge: the residual is the whole dLoss/dDFV[i]
        assert np.allclose(o.residual(i), gd[i], rtol=1e-10, atol=1e-14)


def test_textbook_special_case_one_distinct_image_per_view():
    """All images distinct, one per view, M = 1: the ready list is the batch's dLoss/dDFV rows."""
    rng = np.random.default_rng(5)
    o = small_oracle(rng, M=1)
    batch = batch_from_lists([0, 1, 2, 3], [0, 1, 2, 3], [[8], [3], [5], [0]], [1, 0, 1, 0])
    before = copy.deepcopy(o)
    _, _, _, gd, _, _ = _torch_step(before, batch, 0.0)
    r = o.step(batch, 0.0)
    assert r.ready_ids.tolist() == [0, 3, 5, 8]
    assert np.allclose(r.ready_grads, gd[[0, 3, 5, 8]], rtol=1e-10, atol=1e-14)


# ------------------------------------------------------------------ invariants of the bookkeeping
@pytest.mark.parametrize("M", [1, 2, 3, 5])
def test_store_invariants_over_steps(M):
    rng = np.random.default_rng(10 + M)
    o = small_oracle(rng, n_images=6, M=M)
    occurrences = {i: [] for i in range(6)}          # every per-occurrence gradient, in arrival order
    emitted = {i: [] for i in range(6)}
    for step in range(5):
        batch = random_batch(rng, 9, 7, 5, 6, max_images=4, allow_empty=True)
        r = o.step(batch, 0.05)
        # (v) a view's occurrence gradients sum to its pooled-slot gradient
        for b in range(batch.B):
            sl = slice(batch.img_off[b], batch.img_off[b + 1])
            if sl.stop > sl.start:
                assert np.allclose(r.occ_grads[sl].sum(0), r.dx[b, 2 * o.d:], rtol=1e-12, atol=1e-16)
        for j, i in enumerate(batch.img_id.tolist()):
            occurrences[i].append(r.occ_grads[j])
        # ready list is ordered by image id; emissions of one image keep their order
        assert r.ready_ids.tolist() == sorted(r.ready_ids.tolist())
        for i, g in zip(r.ready_ids.tolist(), r.ready_grads):
            emitted[i].append(g)
        for i in range(6):
            n = len(occurrences[i])
            assert o.counts.get(i, 0) == n                               # (i)
            assert len(emitted[i]) == n // M                             # (ii)
            for k, g in enumerate(emitted[i]):                           # k-th emission = mean of k-th M
                assert np.allclose(g, np.mean(occurrences[i][k * M:(k + 1) * M], axis=0), rtol=1e-12, atol=1e-16)
            total = np.sum(occurrences[i], axis=0) if n else np.zeros(o.D)
            got = M * np.sum(emitted[i], axis=0) + o.residual(i) if emitted[i] else o.residual(i)
            assert np.allclose(got, total, rtol=1e-12, atol=1e-15)       # (iii) conservation
        if M == 1:                                                       # (vi)
            assert r.ready_ids.tolist() == sorted(batch.img_id.tolist())


def test_image_reaching_M_once_emits_mean_of_first_M():
    rng = np.random.default_rng(20)
    o = small_oracle(rng, M=3)
    batch = batch_from_lists([0, 1, 2, 3], [0, 0, 1, 1], [[2, 5], [2], [2, 5], [2]], [1, 0, 0, 1])
    r = o.step(batch, 0.0)
    occ_of_2 = r.occ_grads[[0, 2, 3, 5]]
    assert r.ready_ids.tolist() == [2]
    assert np.allclose(r.ready_grads[0], occ_of_2[:3].mean(0), rtol=1e-13)
    assert np.allclose(o.residual(2), occ_of_2[3], rtol=1e-13) and o.counts[2] == 4 and o.counts[5] == 2


def test_refresh_leaves_store_and_counts_alone():
    rng = np.random.default_rng(21)
    o = small_oracle(rng, M=3)
    o.step(random_batch(rng, 8, 7, 5, 9), 0.1)
    store = copy.deepcopy(o.store)
    counts = dict(o.counts)
    tables = copy.deepcopy((o.user_emb._dense, o.url_emb._dense, o.mlp))
    o.refresh_dfv([1, 4], rng.normal(0, 1, (2, 3)))
    assert counts == o.counts and store.keys() == o.store.keys()
    assert all(np.array_equal(a, b) for k in store for a, b in zip(store[k], o.store[k]))
    assert np.array_equal(tables[0], o.user_emb._dense) and np.array_equal(tables[1], o.url_emb._dense)
    b2 = batch_from_lists([0], [0], [[1]], [1])
    assert np.array_equal(o.step(b2, 0.0).x[0, 4:], o.dfv.row(1))


# ------------------------------------------------------------------ grouping
def test_stable_groups_brute_force():
    rng = np.random.default_rng(30)
    for n in (0, 1, 2, 50):
        keys = rng.integers(0, 7, n).astype(np.int32)
        uniq, segoff, perm = stable_groups(keys)
        assert uniq.tolist() == sorted(set(keys.tolist()))
        pairs = sorted((int(k), p) for p, k in enumerate(keys))       # O(n log n) on (key, position)
        assert perm.tolist() == [p for _, p in pairs]
        for s, k in enumerate(uniq):
            seg = perm[segoff[s]:segoff[s + 1]]
            assert all(keys[p] == k for p in seg) and len(seg) == int((keys == k).sum())


# ------------------------------------------------------------------ precision modes
def test_bf16_mode_equals_exact_mode_on_exactly_representable_data():
    """Small integers and halves survive every bf16 rounding, so both modes must agree bit for bit."""
    rng = np.random.default_rng(40)

    def build(prec):
        r = np.random.default_rng(41)
        ints = lambda *s: r.integers(-2, 3, s).astype(np.float64)
        mlp = [(ints(4, 7), ints(4)), (ints(1, 4), ints(1))]
        return GearOracle(RowStore(5, 2, prec.emb, dense=ints(5, 2)), RowStore(5, 2, prec.emb, dense=ints(5, 2)),
                          RowStore(6, 3, prec.dfv, dense=2 * ints(6, 3)), mlp, 2, prec)
    batch = batch_from_lists([0, 1, 2], [3, 4, 0], [[1, 2], [3], [4, 5]], [1, 0, 1])
    a = build(Precision.exact()).step(batch, 0.0)
    b = build(Precision("bf16", "bf16", "bf16", "f32")).step(batch, 0.0)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.logits, b.logits)


def test_bf16_mode_uses_rounded_weights_forward_and_backward():
    """Master weights that are not bf16 numbers act through their bf16 roundings in both passes.

    One view whose logit is forced to 0 makes dLoss/dz = -1/2 exactly, so with integer data every
    quantity of the backward pass is exact and both precision modes must agree bit for bit."""
    def build(prec, bump, b2=0.0):
        r = np.random.default_rng(43)
        ints = lambda *s: r.integers(-2, 3, s).astype(np.float64)
        nonzero = lambda *s: r.choice([-2.0, -1.0, 1.0, 2.0], s)      # 0 + bump would be a bf16 number
        mlp = [(nonzero(4, 7) + bump, ints(4)), (nonzero(1, 4) + bump, np.array([b2]))]
        return GearOracle(RowStore(5, 2, prec.emb, dense=ints(5, 2)), RowStore(5, 2, prec.emb, dense=ints(5, 2)),
                          RowStore(6, 3, prec.dfv, dense=2 * ints(6, 3)), mlp, 2, prec)
    batch = batch_from_lists([1], [4], [[1, 2]], [1])
    z0 = build(Precision.exact(), 0.0).step(batch, 0.0).logits[0]
    a = build(Precision.exact(), 0.0, -z0).step(batch, 0.0)
    b = build(Precision("bf16", "bf16", "bf16", "f32"), 2.0 ** -12, -z0).step(batch, 0.0)  # bump rounds away
    assert a.logits[0] == 0.0 and b.logits[0] == 0.0 and a.dx.any()
    assert np.array_equal(a.dx, b.dx)
    assert all(np.array_equal(ga[0], gb[0]) and np.array_equal(ga[1], gb[1]) for ga, gb in zip(a.grads, b.grads))
    unrounded = build(Precision.exact(), 2.0 ** -12, -z0).step(batch, 0.0)
    assert not np.array_equal(unrounded.dx, a.dx)


def test_bf16_mode_rounds_operands():
    rng = np.random.default_rng(42)
    o = small_oracle(rng, prec=Precision("bf16", "bf16", "bf16", "f32"))
    r = o.step(random_batch(rng, 5, 7, 5, 9), 0.1)
    assert np.array_equal(r.x, round_bf16(r.x))
    assert not np.array_equal(r.dx[:, 4:], round_bf16(r.dx[:, 4:]))         # dLoss/dx is no operand: not rounded
    assert not np.array_equal(r.dx[:, :4], round_bf16(r.dx[:, :4]))
    assert np.array_equal(o.user_emb._dense, round_bf16(o.user_emb._dense))
    assert all(np.array_equal(W, round_to(W, "f32")) for W, _ in o.mlp)


def test_branch_choice_is_taken_only_within_rounding_distance_of_the_kink():
    """step(relu_choice=...) follows a given ReLU branch only at units whose pre-activation is within
    kink_tol of zero; elsewhere the oracle keeps its own decision and counts the refusal.

    One view, two hidden units: a = [2^-20, 1].  Unit 0 is on by the oracle's own arithmetic but within
    1e-5 of the kink relative to the layer's largest pre-activation; unit 1 is far from it."""
    def build():
        W1 = np.array([[2.0 ** -20, 0.0, 0.0], [0.0, 0.0, 1.0]])
        return GearOracle(RowStore(1, 1, "f64", dense=np.array([[1.0]])), RowStore(1, 1, "f64", dense=np.array([[0.0]])),
                          RowStore(1, 1, "f64", dense=np.array([[1.0]])),
                          [(W1, np.zeros(2)), (np.array([[4.0, -1.0]]), np.array([1.0]))], 1, Precision.exact())
    batch = batch_from_lists([0], [0], [[0]], [1])
    own = build().step(batch, 0.0)
    assert own.dx[0, 0] != 0.0 and own.near_units.tolist() == [0] and np.array_equal(own.dx, own.dx_own)
    on, off = np.array([[True, True]]), np.array([[False, True]])
    same = build().step(batch, 0.0, relu_choice=[on], kink_tol=1e-5)
    assert np.array_equal(same.dx, own.dx) and same.chosen_units == 0 and same.refused_units == 0
    assert same.near_units.tolist() == [1] and same.active_units.tolist() == [2]
    flipped = build().step(batch, 0.0, relu_choice=[off], kink_tol=1e-5)
    # unit 0 off: its delta is zero, so dLoss/dx loses that unit's term; the own-decision result is kept beside it
    assert flipped.chosen_units == 1 and flipped.refused_units == 0
    assert flipped.dx[0, 0] == 0.0 and np.array_equal(flipped.dx_own, own.dx)
    assert np.array_equal(flipped.dx[0, 2:], own.dx[0, 2:]) or abs(flipped.logits[0] - own.logits[0]) < 1e-5
    # the far unit cannot be flipped, whatever the choice says; nor can any unit when kink_tol is 0
    far = build().step(batch, 0.0, relu_choice=[np.array([[True, False]])], kink_tol=1e-5)
    assert far.refused_units == 1 and far.chosen_units == 0 and np.array_equal(far.dx, own.dx)
    none = build().step(batch, 0.0, relu_choice=[off], kink_tol=0.0)
    assert none.refused_units == 1 and np.array_equal(none.dx, own.dx)


def test_a_unit_switched_on_below_zero_passes_zero_forward_and_its_gradient_backward():
    """A chosen "on" at a unit whose own pre-activation is just below zero: ReLU's value there is 0, not the
    negative pre-activation, so the logit is that of the own pass; backward the unit counts as active, so
    dLoss/dx gains its term.  a = [-2^-20, 1], logit weights [4, -1]."""
    W1 = np.array([[-2.0 ** -20, 0.0, 0.0], [0.0, 0.0, 1.0]])
    def build():
        return GearOracle(RowStore(1, 1, "f64", dense=np.array([[1.0]])), RowStore(1, 1, "f64", dense=np.array([[0.0]])),
                          RowStore(1, 1, "f64", dense=np.array([[1.0]])),
                          [(W1, np.zeros(2)), (np.array([[4.0, -1.0]]), np.array([1.0]))], 1, Precision.exact())
    batch = batch_from_lists([0], [0], [[0]], [1])
    own = build().step(batch, 0.0)
    on = build().step(batch, 0.0, relu_choice=[np.array([[True, True]])], kink_tol=1e-5)
    assert on.chosen_units == 1 and own.dx[0, 0] == 0.0
    assert on.logits[0] == own.logits[0] == 0.0 and on.loss == own.loss          # z = 4 * 0 - 1 * 1 + 1
    dz = 0.5 - 1.0                                                               # sigmoid(0) - y, one view
    assert on.dx[0, 0] == dz * 4.0 * W1[0, 0] and np.array_equal(on.dx[0, 1:], own.dx[0, 1:])


def test_branch_choice_decides_what_the_step_applies():
    """The state after a step follows the chosen branches (weights, rows, stored gradients), so that two
    arithmetics that agree on the branches stay together over many steps."""
    rng = np.random.default_rng(8)
    a, b = small_oracle(rng), small_oracle(np.random.default_rng(8))
    batch = random_batch(np.random.default_rng(9), 6, 7, 5, 9)
    ra = a.step(batch, 0.1)
    # every unit declared ambiguous (kink_tol above 1) and the opposite branch asked for at one active
    # unit of the first hidden layer; the layers above are given the branches that follow from it
    choice, x, flipped_unit = [], ra.x, None
    for l in range(len(a.mlp) - 1):
        pre = x @ b.mlp[l][0].T + b.mlp[l][1]
        act = pre > 0
        if l == 0:
            flipped_unit = tuple(np.argwhere(act)[0])
            act[flipped_unit] = False
        choice.append(act)
        x = np.where(act, pre, 0.0)
    v, u = flipped_unit
    rb = b.step(batch, 0.1, relu_choice=choice, kink_tol=2.0)
    assert rb.chosen_units == 1 and not np.array_equal(rb.dx[v], ra.dx[v]) and np.array_equal(rb.dx_own, ra.dx)
    assert not np.array_equal(a.mlp[0][0][u], b.mlp[0][0][u])                # the unit's weight row saw another gradient
    others = [w for w in range(batch.B) if w != v]
    assert np.array_equal(rb.dx[others], ra.dx[others])
    assert not np.array_equal(a.user_emb.row(batch.user_id[v]), b.user_emb.row(batch.user_id[v]))


# ------------------------------------------------------------------ workload recipe
def test_workload_batches_are_reproducible_and_in_range():
    wl = get_workload("tiny")
    src = PageViewSource(wl)
    a, b = src.batch(3), src.batch(3)
    assert all(np.array_equal(getattr(a, f), getattr(b, f)) for f in ("user_id", "url_id", "img_off", "img_id", "label"))
    assert not np.array_equal(a.user_id, src.batch(4).user_id)
    assert a.B == 512 and a.img_off[0] == 0 and a.img_off[-1] == a.nnz
    n = np.diff(a.img_off)
    assert n.min() >= 1 and n.max() <= wl.max_images
    assert 0 <= a.user_id.min() and a.user_id.max() < wl.n_users and a.img_id.max() < wl.n_images
    assert set(np.unique(a.label)) <= {0.0, 1.0}


def test_zipf_ids_follow_the_law():
    from gear_inputs.pageviews import ZipfIds
    z = ZipfIds(1000, 1.1, salt=3)
    rng = np.random.default_rng(0)
    r = z.ranks(rng, 200_000)
    H = np.sum(np.arange(1, 1001) ** -1.1)
    for rank in (0, 1, 9):
        assert abs((r == rank).mean() - (rank + 1) ** -1.1 / H) < 0.01
    ids = z.rank_to_id(np.arange(1000))
    assert sorted(ids.tolist()) == list(range(1000))                  # bijection


def test_oracle_from_seed_uses_lazy_rows():
    wl = get_workload("small")
    o = GearOracle.from_seed(wl.seed, wl.n_users, wl.n_urls, wl.n_images, wl.emb_dim, wl.dfv_dim,
                             wl.layers, wl.M, Precision("f32", "f32", "f32", "f32"))
    batch = PageViewSource(wl).batch(0, batch=64)
    r = o.step(batch, wl.lr)
    assert np.isfinite(r.loss) and 0.3 < r.loss < 1.5
    assert len(o.user_emb._rows) == len(set(batch.user_id.tolist()))
    assert abs(np.std(o.dfv.rows(batch.img_id[:50])) - 1.0) < 0.05
    assert abs(np.std(o.mlp[0][0]) - math.sqrt(2 / 320)) / math.sqrt(2 / 320) < 0.02


def test_epoch_pattern_shows_every_image_once_per_epoch():
    """The "epoch" workload walks a fixed shuffle of the image set: no image twice before all were seen."""
    from gear_inputs import PageViewSource, get_workload
    wl = get_workload("epoch").scaled(batch=300, n_images=1200)
    src = PageViewSource(wl)
    seen = np.concatenate([src.batch(t).img_id for t in range(8)])          # two epochs of four steps
    assert src.batch(0).nnz == 300 and np.array_equal(src.batch(3).img_off, np.arange(301))
    for epoch in (seen[:1200], seen[1200:]):
        assert np.array_equal(np.sort(epoch), np.arange(1200))
    assert np.array_equal(seen[:1200], seen[1200:])                          # the same order every epoch
    assert not np.array_equal(np.sort(seen[:300]), np.arange(300))          # shuffled, not 0..B-1


def test_epoch_pattern_closes_groups_only_after_M_epochs():
    from gear_inputs import PageViewSource, get_workload
    from oracle.from_workload import oracle_for
    wl = get_workload("epoch").scaled(batch=40, n_images=80, M=3, dfv_dim=8, emb_dim=8, layers=(8, 1))
    orc, src = oracle_for(wl), PageViewSource(wl)
    emitted = [len(orc.step(src.batch(t), 0.01).ready_ids) for t in range(8)]  # an epoch is two steps
    assert emitted == [0, 0, 0, 0, 40, 40, 0, 0]


def test_expiry_lists_old_requested_rows_once_and_ascending():
    """Expiry (Section 1, second point): requested and at least `expiry` old, each id once, ascending."""
    o = small_oracle(np.random.default_rng(3))
    n = o.dfv.n_rows
    assert o.expired([], now=5, expiry=0) == []
    assert o.expired([4, 1, 4, 2], now=0, expiry=0) == [1, 2, 4]          # age 0 >= 0: everything asked for
    assert o.expired([4, 1, 4, 2], now=2, expiry=3) == []                   # never stamped = time 0: age 2 < 3
    assert o.expired([4, 1, 4, 2], now=3, expiry=3) == [1, 2, 4]            # age == expiry counts as expired
    o.stamp([1, 4], now=3)
    assert o.expired([4, 1, 4, 2], now=5, expiry=3) == [2]                  # 1 and 4 are 2 old, 2 is 5 old
    assert o.expired([4, 1, 4, 2], now=6, expiry=3) == [1, 2, 4]
    assert o.expired([0], now=6, expiry=3) == [0]                            # only what the batch asks for is listed
    with pytest.raises(ValueError):
        o.expired([n], now=1, expiry=0)
    with pytest.raises(ValueError):
        o.expired([-1], now=1, expiry=0)
    # stamping changes neither gradients nor counters
    before = (dict(o.counts), {k: [g.copy() for g in v] for k, v in o.store.items()})
    o.stamp(range(n), now=9)
    assert before[0] == o.counts and all(np.array_equal(a, b) for k in before[1] for a, b in zip(before[1][k], o.store[k]))


def test_adam_matches_the_library_optimisers():
    """Adam of the Sparse Part (Section 4.1) against torch.optim.Adam (MLP) and torch.optim.SparseAdam
    (tables: only touched rows move, global step in the bias corrections), fed the oracle's gradients."""
    import torch
    rng = np.random.default_rng(11)
    o = small_oracle(rng, n_users=6, n_urls=5)
    # an eps large enough that where it enters the formula matters
    b1, b2, eps, lr = float(np.float32(0.9)), float(np.float32(0.999)), float(np.float32(1e-4)), 0.05
    o.use_adam(b1, b2, eps)
    dense = [torch.tensor(a.copy(), dtype=torch.float64, requires_grad=True) for W, b in o.mlp for a in (W, b)]
    tables = [torch.tensor(o.user_emb._dense.copy(), dtype=torch.float64, requires_grad=True),
              torch.tensor(o.url_emb._dense.copy(), dtype=torch.float64, requires_grad=True)]
    opt_dense = torch.optim.Adam(dense, lr=lr, betas=(b1, b2), eps=eps)
    opt_rows = torch.optim.SparseAdam(tables, lr=lr, betas=(b1, b2), eps=eps)
    d = o.d
    untouched_once = False
    for step in range(4):
        batch = random_batch(rng, 3, 6, 5, 9)                  # few views: some rows are skipped in a step
        r = o.step(batch, lr)
        for p, gnp in zip(dense, [a for dW, db in r.grads for a in (dW, db)]):
            p.grad = torch.tensor(np.asarray(gnp, dtype=np.float64).reshape(p.shape))
        opt_dense.step()
        for p, ids, lo in ((tables[0], batch.user_id, 0), (tables[1], batch.url_id, d)):
            uniq = sorted(set(int(i) for i in ids))
            untouched_once |= len(uniq) < p.shape[0]
            vals = np.stack([sum(r.dx[k, lo:lo + d] for k in range(batch.B) if int(ids[k]) == u) for u in uniq])
            p.grad = torch.sparse_coo_tensor(torch.tensor([uniq]), torch.tensor(vals), p.shape).coalesce()
        # SparseAdam writes the same update as lr sqrt(1-b2^t)/(1-b1^t) m / (sqrt(v) + eps'), eps' = eps sqrt(1-b2^t)
        opt_rows.param_groups[0]["eps"] = eps * math.sqrt(1.0 - b2 ** (step + 1))
        opt_rows.step()
        got = [a for W, b in o.mlp for a in (W, b)] + [o.user_emb._dense, o.url_emb._dense]
        for mine, ref in zip(got, dense + tables):
            ref = ref.detach().numpy().reshape(mine.shape)
            assert np.abs(mine - ref).max() <= 2e-6 * max(np.abs(ref).max(), lr), step   # moments are kept in fp32
    assert untouched_once


def test_adam_first_step_moves_every_element_by_the_rate():
    """Closed form: at t = 1 the update is lr * g / (|g| + eps'), i.e. +-lr where |g| >> eps."""
    rng = np.random.default_rng(5)
    o = small_oracle(rng)
    before = [(W.copy(), b.copy()) for W, b in o.mlp]
    o.use_adam()
    r = o.step(random_batch(rng, 6, 7, 5, 9), 1e-3)
    for (W0, b0), (W1, b1), (dW, db) in zip(before, o.mlp, r.grads):
        big = np.abs(dW) > 1e-4
        assert big.any()
        assert np.allclose((W0 - W1)[big], 1e-3 * np.sign(dW)[big], rtol=1e-3)
    # plain SGD is untouched by the new code path
    p = small_oracle(np.random.default_rng(5))
    q = small_oracle(np.random.default_rng(5))
    bt = random_batch(np.random.default_rng(6), 6, 7, 5, 9)
    rp = p.step(bt, 0.1)
    assert all(np.array_equal(W0 - 0.1 * dW, W1) for (W0, _), (W1, _), (dW, _) in zip(q.mlp, p.mlp, rp.grads))


def test_dense_standin_gradient_is_the_chain_rule_of_eq1():
    """Eq. 1: dLoss/dWd = dLoss/dDFV * dDFV/dWd.  With M = 1 every occurrence is emitted at once, so the
    stand-in's weight change over one step is -lr times the derivative of the Sparse Part's loss with
    respect to Wd when the cache holds Wd raw[i]; checked by central finite differences on the loss."""
    from oracle.dense_standin import DenseStandIn
    rng = np.random.default_rng(21)
    n_images, D, r = 9, 3, 4
    raw, wd0 = rng.normal(0, 1, (n_images, r)), rng.normal(0, 0.5, (D, r))

    batch = random_batch(np.random.default_rng(5), 6, 7, 5, n_images)
    o = small_oracle(np.random.default_rng(77), n_images=n_images, D=D, M=1)
    dense = DenseStandIn(raw, wd0, "f64")
    dense.raw, dense.wd = np.asarray(raw, np.float64), np.asarray(wd0, np.float64)   # unrounded, for the check
    o.refresh_dfv(range(n_images), dense.infer(range(n_images)))
    res = o.step(batch, 0.0)
    before = dense.wd.copy()
    dense.backward(res.ready_ids, res.ready_grads, 1.0)
    analytic = before - dense.wd                                      # lr = 1: the gradient itself (fp32-rounded)
    h = 1e-6
    for (a, b) in [(0, 0), (1, 2), (2, 3), (0, 1)]:
        vals = []
        for sgn in (+1, -1):
            wd = np.array(wd0, dtype=np.float64)
            wd[a, b] += sgn * h
            oo = small_oracle(np.random.default_rng(77), n_images=n_images, D=D, M=1)
            oo.refresh_dfv(range(n_images), np.asarray(raw, np.float64) @ wd.T)
            vals.append(oo.step(batch, 0.0).loss)
        numeric = (vals[0] - vals[1]) / (2 * h)
        assert abs(numeric - analytic[a, b]) <= 1e-6 * max(1.0, abs(numeric)) + 1e-7, (a, b, numeric, analytic[a, b])
    # the steps per emission add up to one step with the summed outer products
    total = sum(np.outer(g, raw[int(i)]) for i, g in zip(res.ready_ids, res.ready_grads))
    assert np.allclose(analytic, total, rtol=0, atol=1e-6 * np.abs(total).max() + 1e-7)


def test_dense_standin_infer_rounds_to_the_cache_type():
    from oracle.dense_standin import DenseStandIn
    rng = np.random.default_rng(2)
    dense = DenseStandIn(rng.normal(0, 1, (5, 8)), rng.normal(0, 1, (3, 8)), "bf16")
    rows = dense.infer([4, 0, 4])
    assert np.array_equal(rows, round_bf16(rows)) and np.array_equal(rows[0], rows[2])
    assert np.allclose(rows[1], dense.wd @ dense.raw[0], rtol=2 ** -8)
    with pytest.raises(ValueError):
        dense.infer([5])


def test_dense_standin_weights_stay_fp32_values():
    """The stand-in's weights are fp32 masters: one rounding after a backward pass over a whole ready list,
    none between its emissions.  Wd = [[1]], raw = [[1], [1]], two emissions of -2^-24 at lr 1: each alone is
    half a unit in the last place of 1 and would round back to 1 (ties to even); together they are one."""
    from oracle.dense_standin import DenseStandIn
    dense = DenseStandIn(np.array([[1.0], [1.0]]), np.array([[1.0]]), "f32")
    g = np.array([[-2.0 ** -24], [-2.0 ** -24]])
    dense.backward([0, 1], g, 1.0)
    assert dense.wd[0, 0] == 1.0 + 2.0 ** -23 == float(np.float32(dense.wd[0, 0]))
    dense = DenseStandIn(np.array([[1.0], [1.0]]), np.array([[1.0]]), "f32")
    dense.backward([0], g[:1], 1.0)
    assert dense.wd[0, 0] == 1.0                                  # 1 + 2^-24 is not an fp32 number
