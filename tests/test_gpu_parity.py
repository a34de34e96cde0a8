"""Parity of the HIP path (through the C ABI) with the CPU oracle, on a real MI355X.

Integer results are compared bit for bit, floating point by the row rule of oracle/compare.py
(1e-5 relative for fp32 workloads, 2e-2 for bf16).  Both sides start from their own counter-based
initialiser and run freely; nothing the oracle consumes comes from the GPU.
"""
import math
import os

import numpy as np
import pytest
import torch

from gear_inputs import PageViewSource, get_workload
from gear_inputs.pageviews import PageViewBatch, batch_from_lists
from oracle import philox_normal
from oracle.compare import REL, assert_delta_rows_close, assert_rows_close, row_errors
from oracle.from_workload import oracle_for
from oracle.gear_oracle import stable_groups
from oracle.rounding import round_to

pytestmark = pytest.mark.gpu

g = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global g
    import paper_1806_03925_amd as mod
    assert torch.cuda.is_available(), "these tests need the GPU"
    g = mod
    yield


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def make_pair(wl, max_batch=None, ready_cap=None):
    cfg = g.config_for(wl, max_batch=max_batch)
    st = g.GearState(cfg, debug=True, ready_cap=ready_cap)
    g.gear_init_tables(st)
    g.gear_fill_normal(st.dfv_cache, wl.n_images, wl.dfv_dim, wl.seed, 3, wl.dfv_std)
    return cfg, st, oracle_for(wl)


# A hidden unit whose pre-activation is within this fraction of its layer's largest one may land on
# either side of the ReLU kink: fp32 products summed in another order differ by about 1e-6 of the
# layer's scale; with bf16 operands an element of x or h can round to the neighbouring bf16 value
# (2^-8 relative), which shifts the next layer's pre-activations by about 1e-3 of their scale.
KINK_TOL = {"f32": 1e-5, "bf16": 2e-3}
# A unit taking the other branch moves a view's dLoss/dx row by about 1/sqrt(active units) of its scale;
# a row compared with the oracle's own decisions may be off by this multiple of (units of the view
# that took the other branch) / sqrt(active units), and no more.
KINK_C = 4.0
STATS = []          # one line per comparison: how close to the bars and caps each test runs


def note(line):
    STATS.append(line)
    print("[parity] " + line, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _stats_file():
    yield
    out = os.environ.get("GEAR_PARITY_MARGINS")      # a file to keep the lines in
    if STATS and out:
        with open(out, "w") as f:
            f.write("\n".join(STATS) + "\n")


class Pair:
    """The HIP path and the oracle side by side, both from their own initial state, free-running.

    Every step is compared twice.  (1) Against the oracle's own ReLU decisions: dLoss/dx rows of views
    with no hidden unit near the kink must pass the row rule; the others may differ, by at most
    KINK_C * (units on the other branch) / sqrt(active units) of the row's scale, and only a capped
    number of them do.  (2) Against
    the oracle taking, at near-kink units only, the branch the kernels took (read from the stored
    activations): then every output and every touched row of the state must pass the row rule, with no
    exemption.  The oracle checks the distance to the kink itself and refuses a branch elsewhere; a
    refusal fails the test.  The oracle's state advances with (2), so both sides stay on the same
    branches over many steps."""

    def __init__(self, wl, max_batch=None, ready_cap=None, adam_eps=None):
        self.wl = wl
        self.cfg, self.st, self.orc = make_pair(wl, max_batch=max_batch, ready_cap=ready_cap)
        self.rel = REL[wl.mlp_dtype]
        self.kink_tol = KINK_TOL[wl.mlp_dtype]
        self.adam = None
        if adam_eps is not None:
            self.orc.use_adam(eps=adam_eps)
            self.adam = g.AdamMoments(self.st, eps=adam_eps)
        self.steps = 0
        self.term = {}                                   # (table, id) -> largest |lr * gradient term| summed into the row
        self.before = {"user": {}, "url": {}}            # id -> (kernel's row, oracle's row) before their first touch
        torch.cuda.synchronize()
        self.mlp_before = (f64(self.st.mlp_params), [(W.copy(), b.copy()) for W, b in self.orc.mlp])
        self.flip_total = 0

    def _snapshot(self, batch):
        for name, table, store, ids in (("user", self.st.user_emb, self.orc.user_emb, batch.user_id),
                                        ("url", self.st.url_emb, self.orc.url_emb, batch.url_id)):
            seen = self.before[name]
            new = np.array(sorted(set(ids.tolist()) - seen.keys()), dtype=np.int64)
            if len(new):
                got = f64(table[torch.from_numpy(new).cuda()])
                ref = store.rows(new)
                for k, a, b in zip(new.tolist(), got, ref):
                    seen[k] = (a.copy(), b.copy())

    def step(self, batch: PageViewBatch, lr: float, what: str, flip_cap=None):
        """Run one step on both sides and compare every output; returns the oracle's result."""
        wl, st, rel = self.wl, self.st, self.rel
        self._snapshot(batch)
        dev = g.DeviceBatch.from_host(batch)
        if self.adam is None:
            g.gear_step(st, dev, wl.M, lr)
        else:
            g.gear_step_adam(st, dev, wl.M, lr, self.adam)
        torch.cuda.synchronize()
        B, d = batch.B, wl.emb_dim
        assert int(st.status.item()) == 0, what
        choice = [(st.region(f"h{l}", B) > 0).cpu().numpy() for l in range(len(wl.layers) - 1)]
        lr32 = float(np.float32(lr))
        ref = self.orc.step(batch, lr32, relu_choice=choice, kink_tol=self.kink_tol)
        self.steps += 1
        for key, t in ref.emb_term_scale.items():
            self.term[key] = max(self.term.get(key, 0.0), lr32 * t)
        assert ref.refused_units == 0, \
            f"{what}: {ref.refused_units} hidden units took another branch than the oracle away from the kink"

        # grouping of the image ids
        nu = int(st.dbg[3].item())
        assert nu == len(ref.img_unique), what
        assert np.array_equal(st.dbg[0][:nu].cpu().numpy(), ref.img_unique), what
        assert np.array_equal(st.dbg[1][:nu + 1].cpu().numpy(), ref.img_segoff), what
        assert np.array_equal(st.dbg[2][:batch.nnz].cpu().numpy(), ref.img_perm), what

        # forward
        wx = assert_rows_close(f64(st.region("x", B)), ref.x, rel, f"{what}: x")
        wz = assert_rows_close(f64(st.region("logits", B)), ref.logits, rel, f"{what}: logits")
        assert abs(float(st.loss.item()) - ref.loss) <= rel * abs(ref.loss), (what, st.loss.item(), ref.loss)

        # (1) dLoss/dx against the oracle's own decisions
        dx = f64(st.region("dx", B))
        err, scale = row_errors(dx, ref.dx_own)
        off = err > rel * scale
        near = ref.near_units > 0
        assert not (off & ~near).any(), \
            f"{what}: dx rows off with no unit near a kink: {np.flatnonzero(off & ~near)[:5]}"
        bound = KINK_C * ref.chosen_per_view / np.sqrt(np.maximum(ref.active_units, 1))
        assert (err[off] <= bound[off] * scale[off]).all(), \
            f"{what}: a dx row is off by more than {KINK_C} * (units on the other branch) / sqrt(active units)"
        worst_flip = float((err[off] / np.maximum(bound[off] * scale[off], 1e-300)).max()) if off.any() else 0.0
        cap = max(2, 0.002 * B) if wl.mlp_dtype == "f32" else max(2, 0.06 * B)
        if flip_cap is not None:
            cap = max(2, flip_cap * B)
        assert off.sum() <= cap, f"{what}: {off.sum()} of {B} dx rows differ at kinks ({near.sum()} rows are near one)"
        assert np.median(err / scale) <= rel / 4, f"{what}: median dx row error {np.median(err / scale):.2e}"
        self.flip_total += int(off.sum())

        # (2) the same branches on both sides: everything by the row rule, nothing exempt
        wdx = assert_rows_close(dx, ref.dx, rel, f"{what}: dx (same branches)")
        n_ready = int(st.n_ready.item())
        assert n_ready == len(ref.ready_ids), what
        assert np.array_equal(st.ready_ids[:n_ready].cpu().numpy(), ref.ready_ids), what
        wr = 0.0
        if n_ready:
            wr = assert_rows_close(f64(st.ready_grads[:n_ready]), ref.ready_grads, rel, f"{what}: ready_grads",
                                   term_scale=ref.ready_term_scale)
        note(f"{what}: B {B}, rows near a kink {int(near.sum())}, rows differing under own decisions {int(off.sum())} "
             f"(cap {int(cap)}; worst {worst_flip:.2f} of its bound), units given the kernel's branch {ref.chosen_units}; worst error / bar: x {wx / rel:.3f}, "
             f"logits {wz / rel:.3f}, dx {wdx / rel:.3f}, ready_grads ({n_ready} rows) {wr / rel:.3f}")
        return ref

    def check_state(self, what, changes=True, resolution=None):
        """The persistent state: counters bit for bit, accumulators by rows, and what the steps changed
        in the tables and the MLP as a change (after - before on both sides).  resolution: the median
        row's change must be at least this many times what the comparison allows it to be off by (above
        1, a step that left the rows as they were puts more than half of them outside the allowance)."""
        wl, st, orc, rel = self.wl, self.st, self.orc, self.rel
        counts = st.counts.cpu().numpy()
        touched = np.array(sorted(orc.counts), dtype=np.int64)
        assert int(counts.sum()) == sum(orc.counts.values()), what
        assert np.array_equal(counts[touched], np.array([orc.counts[i] for i in touched], dtype=np.int32)), what
        wa = 0.0
        if len(touched):
            acc = f64(st.grad_accum[torch.from_numpy(touched).cuda()])
            ref = np.stack([orc.residual(i) for i in touched])
            # images whose count is a multiple of M hold exactly zero
            full = np.array([orc.counts[i] % wl.M == 0 for i in touched])
            assert not acc[full].any(), what
            wa = assert_rows_close(acc, ref, rel, f"{what}: grad_accum",
                                   term_scale=[orc.residual_term_scale(i) for i in touched])
        # untouched accumulators are still zero
        nz_rows = int((st.grad_accum != 0).any(dim=1).sum().item())
        assert nz_rows <= len(touched), what
        line = f"{what}: {len(touched)} accumulator rows, worst error / bar {wa / rel:.3f}"
        if not changes:
            note(line)
            return
        for name, table, store in (("user", st.user_emb, orc.user_emb), ("url", st.url_emb, orc.url_emb)):
            seen = self.before[name]
            ids = np.array(sorted(seen), dtype=np.int64)
            if len(ids):
                got = f64(table[torch.from_numpy(ids).cuda()])
                worst, res = assert_delta_rows_close(
                    got, np.stack([seen[k][0] for k in ids.tolist()]), store.rows(ids),
                    np.stack([seen[k][1] for k in ids.tolist()]), rel, wl.emb_dtype, self.steps, f"{what}: {name}_emb",
                    term_scale=[self.term[(name, k)] for k in ids.tolist()])
                line += f"; {name}_emb {len(ids)} rows: worst error / allowance {worst:.3f}, median change / allowance {res:.1f}"
                if resolution is not None and wl.emb_dtype == "f32":
                    assert res >= resolution, f"{what}: {name}_emb changes are not resolved ({res:.2f})"
        gpu_before, ref_before = self.mlp_before
        for l, (W, b) in enumerate(orc.mlp):
            Wg, bg = st.layer_params(l)
            wo, bo = g.gear_mlp_param_offset(self.cfg, l, 0), g.gear_mlp_param_offset(self.cfg, l, 1)
            worst, res = assert_delta_rows_close(f64(Wg), gpu_before[wo:wo + W.size].reshape(W.shape), W,
                                                 ref_before[l][0], rel, "f32", self.steps, f"{what}: W{l}")
            wb, _ = assert_delta_rows_close(f64(bg), gpu_before[bo:bo + b.size], b, ref_before[l][1], rel, "f32",
                                            self.steps, f"{what}: b{l}")
            line += f"; W{l} {worst:.3f} (change / allowance {res:.1f}), b{l} {wb:.3f}"
            if resolution is not None:
                assert res >= resolution, f"{what}: W{l} changes are not resolved ({res:.2f})"
        note(line)


# ------------------------------------------------------------------ initialiser
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fill_normal_matches_generator_bit_for_bit(dtype):
    rows, dim, seed, stream, std = 3001, 72, 0x1234_5678_9ABC_DEF0, 5, 0.37
    t = torch.empty((rows, dim), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    g.gear_fill_normal(t, rows, dim, seed, stream, std)
    torch.cuda.synchronize()
    ref = round_to(philox_normal.normal_rows(seed, stream, np.arange(rows), dim, std).astype(np.float64), dtype)
    assert np.array_equal(f64(t), ref)


def test_init_tables_matches_oracle_state():
    wl = get_workload("tiny")
    cfg, st, orc = make_pair(wl)
    torch.cuda.synchronize()
    assert np.array_equal(f64(st.user_emb), orc.user_emb.rows(np.arange(wl.n_users)))
    assert np.array_equal(f64(st.url_emb[:100]), orc.url_emb.rows(np.arange(100)))
    assert np.array_equal(f64(st.dfv_cache[-50:]), orc.dfv.rows(np.arange(wl.n_images - 50, wl.n_images)))
    for l, (W, b) in enumerate(orc.mlp):
        Wg, bg = st.layer_params(l)
        assert np.array_equal(f64(Wg), W) and not bg.any()
    assert not st.grad_accum.any() and not st.counts.any()


# ------------------------------------------------------------------ grouping
@pytest.mark.parametrize("n,key_range", [(0, 10), (1, 10), (5, 3), (2048, 50), (2049, 1 << 26), (6000, 1),
                                         (50_000, 4_000_000), (50_000, 700), (131_072, 50_000_000)])
def test_group_ids_matches_brute_force(n, key_range):
    wl = get_workload("tiny").scaled(batch=max(n, 1), max_images=1)
    cfg = g.config_for(wl)
    st = g.GearState(cfg)
    rng = np.random.default_rng(n + key_range)
    keys = rng.integers(0, key_range, n).astype(np.int32)
    if n > 100:
        keys[rng.integers(0, n, n // 3)] = keys[0]            # one long segment
    unique, segoff, perm, n_unique = g.gear_group_ids(st, torch.from_numpy(keys).cuda(), key_range)
    torch.cuda.synchronize()
    ru, rs, rp = stable_groups(keys)
    nu = int(n_unique.item())
    assert nu == len(ru)
    assert np.array_equal(unique[:nu].cpu().numpy(), ru)
    assert np.array_equal(segoff[:nu + 1].cpu().numpy(), rs)
    assert np.array_equal(perm[:n].cpu().numpy(), rp)


# ------------------------------------------------------------------ full steps
def test_tiny_all_steps_free_running():
    wl = get_workload("tiny")
    pair = Pair(wl)
    src = PageViewSource(wl)
    emitted = 0
    for step in range(wl.steps):
        ref = pair.step(src.batch(step), wl.lr, f"tiny step {step}")
        emitted += len(ref.ready_ids)
        pair.check_state(f"tiny after step {step}")
    assert emitted > 0 and pair.flip_total == 0


@pytest.mark.parametrize("name,batch,steps,lr", [
    ("small", 1000, 3, 0.01),        # ragged batch: 1000 = 7 * 128 + 104 views
    ("small", 4096, 2, 2.0),         # large rate so that embedding updates are far above rounding
    ("hotkey", 2500, 3, 0.01),       # windows crossing M several times per step
    ("bf16", 1500, 3, 0.01),
    ("bf16", 4096, 1, 4.0),         # one step at a rate that lifts bf16 row updates above their rounding
    ("large", 700, 2, 0.01),
])
def test_workload_steps_free_running(name, batch, steps, lr):
    wl = get_workload(name)
    if name in ("bf16", "large"):                      # keep the oracle's tables small
        wl = wl.scaled(n_users=200_000, n_urls=1 << 18, n_images=20_000)
    if name == "hotkey":
        wl = wl.scaled(n_images=300)                     # many images pass M = 64 more than once per step
    pair = Pair(wl, max_batch=batch)
    src = PageViewSource(wl)
    for step in range(steps):
        pair.step(src.batch(step, batch=batch), lr, f"{name} B={batch} step {step}")
        pair.check_state(f"{name} B={batch} after step {step}")
    assert sum(pair.orc.counts.values()) > 0


@pytest.mark.parametrize("dtype,hidden", [
    ("f32", (64, 512)),      # last hidden width 512 fp32: 128 16-byte pieces per row, two per lane
    ("f32", (32, 1024)),     # 1024 fp32: four pieces per lane (the widest the logit layer takes)
    ("bf16", (64, 1024)),    # 1024 bf16: two pieces per lane
    ("bf16", (64, 8)),       # a single piece: most lanes of a group idle
])
def test_wide_and_narrow_last_hidden_layer(dtype, hidden):
    """The logit/loss kernel picks lanes per view and pieces per lane from the last hidden width."""
    wl = get_workload("tiny").scaled(layers=(*hidden, 1), mlp_dtype=dtype, emb_dtype=dtype, dfv_dtype=dtype)
    pair = Pair(wl)
    src = PageViewSource(wl)
    for step in range(2):
        pair.step(src.batch(step, batch=389), 0.05, f"{dtype} hidden {hidden} step {step}")
    pair.check_state(f"{dtype} hidden {hidden}")


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_a_product_made_in_two_column_parts_has_the_same_bits(dtype):
    """A step makes dLoss/dx either as one product or as two (embedding slots, DFV slot), depending on
    its size: an element must not depend on which tile of which launch it falls into."""
    gen = torch.Generator().manual_seed(7)
    A = torch.randn(777, 1024, generator=gen).to(dtype).cuda()
    W = (torch.randn(1152, 1024, generator=gen) / 32).to(dtype).cuda()     # rows = columns of the result
    whole = g.gear_gemm(A, W, 0)
    left = g.gear_gemm(A, W[:128].contiguous(), 0)
    right = g.gear_gemm(A, W[128:].contiguous(), 0)
    torch.cuda.synchronize()
    assert torch.equal(whole[:, :128], left) and torch.equal(whole[:, 128:], right)


@pytest.mark.parametrize("batch", [1056, 389])
def test_three_hidden_layers(batch):
    """Weight gradients of all hidden layers: in one launch over two ragged ranges of the batch (1056 = 33 * 32
    rows, result tiles of 320 and 72 rows and columns) or, for a batch that is no multiple of the
    k-tile, one launch per layer."""
    wl = get_workload("tiny").scaled(layers=(320, 72, 64, 1), mlp_dtype="bf16", emb_dtype="bf16", dfv_dtype="bf16",
                                     batch=1056)
    pair = Pair(wl)
    src = PageViewSource(wl)
    for step in range(2):
        pair.step(src.batch(step, batch=batch), 0.5, f"three hidden layers B={batch} step {step}")
    pair.check_state(f"three hidden layers B={batch}")


def test_batches_smaller_than_the_largest_take_whichever_weight_gradient_path_fits():
    """A state sized for 1500 views (no multiple of 32 rows) steps through batches of 1472 (all weight
    gradients in one launch, more split-K partials than a layer-by-layer step of 1500 needs), 1500 and 700."""
    wl = get_workload("bf16").scaled(n_users=50_000, n_urls=1 << 15, n_images=5_000, M=4)
    pair = Pair(wl, max_batch=1500)
    src = PageViewSource(wl)
    for step, batch in enumerate((1472, 1500, 700)):
        pair.step(src.batch(step, batch=batch), 0.05, f"max 1500, B={batch}")
    pair.check_state("max 1500")


def test_epoch_pattern_free_running():
    """One image per view, every image once per epoch: cold rows each step, groups close after M epochs."""
    wl = get_workload("epoch").scaled(batch=600, n_images=1800, M=2)
    pair = Pair(wl)
    src = PageViewSource(wl)
    emitted = []
    for step in range(8):                                   # 2 2/3 epochs of three steps
        ref = pair.step(src.batch(step), wl.lr, f"epoch step {step}")
        emitted.append(len(ref.ready_ids))
    pair.check_state("epoch after 8 steps")
    assert emitted == [0, 0, 0, 600, 600, 600, 0, 0]


def test_expired_ids_and_stamps_match_oracle():
    """Expiry of cached inference results: bit-exact lists over several steps of refresh + stamp."""
    wl = get_workload("hotkey").scaled(n_images=3000, batch=700)
    pair = Pair(wl)
    cfg, st, orc = pair.cfg, pair.st, pair.orc
    stamp = torch.zeros(wl.n_images, dtype=torch.int32, device="cuda")
    src = PageViewSource(wl)
    total = 0
    for now, expiry in [(0, 1), (1, 1), (2, 3), (3, 3), (4, 2), (5, 0), (9, 4)]:
        b = src.batch(now)
        ids = torch.from_numpy(b.img_id).cuda()
        out, n_out = g.gear_expired_ids(st, ids, stamp, now, expiry)
        torch.cuda.synchronize()
        ref = orc.expired(b.img_id, now, expiry)
        n = int(n_out.item())
        assert int(st.status.item()) == 0 and n == len(ref), (now, expiry, n, len(ref))
        assert np.array_equal(out[:n].cpu().numpy(), np.asarray(ref, dtype=np.int32)), (now, expiry)
        # the caller recomputes those rows (here: fresh random rows), writes and stamps them
        if n:
            rows = torch.randn(n, wl.dfv_dim, device="cuda")
            g.gear_refresh_dfv(st, out[:n], rows)
            g.gear_stamp_dfv(st, stamp, out[:n], now)
            orc.refresh_dfv(ref, rows.double().cpu().numpy())
            orc.stamp(ref, now)
        total += n
    torch.cuda.synchronize()
    assert total > 0
    host = stamp.cpu().numpy()
    assert all(host[i] == t for i, t in orc.stamps.items()) and int((host != 0).sum()) <= len(orc.stamps)
    # refreshed rows are what the next step gathers
    pair.step(src.batch(20), wl.lr, "step after refreshes")
    # empty request, and an id out of range
    out, n_out = g.gear_expired_ids(st, torch.zeros(0, dtype=torch.int32, device="cuda"), stamp, 50, 0)
    torch.cuda.synchronize()
    assert int(n_out.item()) == 0 and int(st.status.item()) == 0
    bad = torch.tensor([1, wl.n_images, 2], dtype=torch.int32, device="cuda")
    out, n_out = g.gear_expired_ids(st, bad, stamp, 50, 0)
    torch.cuda.synchronize()
    assert int(st.status.item()) == g.GEAR_ERR_RANGE and int(n_out.item()) == 0
    g.gear_stamp_dfv(st, stamp, None, 77)                    # all rows
    torch.cuda.synchronize()
    assert int((stamp != 77).sum().item()) == 0


def test_refresh_and_stamp_with_the_count_on_the_device():
    """gear_refresh_dfv_n / gear_stamp_dfv_n against the calls that take the count from the host: same
    cache, same stamps, also when the list is empty and when the device word exceeds the capacity."""
    wl = get_workload("hotkey").scaled(n_images=3000, batch=700)
    src = PageViewSource(wl)
    states = []
    for on_device in (False, True):
        cfg, st, _ = make_pair(wl)
        stamp = torch.zeros(wl.n_images, dtype=torch.int32, device="cuda")
        pool = torch.randn(wl.max_nnz, wl.dfv_dim, generator=torch.Generator().manual_seed(3)).cuda().to(st.dfv_cache.dtype)
        for now, expiry in [(0, 1), (1, 1), (2, 3), (3, 50), (4, 2)]:
            ids = torch.from_numpy(src.batch(now).img_id).cuda()
            out, n_out = g.gear_expired_ids(st, ids, stamp, now, expiry)
            if on_device:
                g.gear_refresh_dfv_n(st, out, pool[: out.numel()], n_out)
                g.gear_stamp_dfv_n(st, stamp, out, n_out, now)
            else:
                n = int(n_out.item())
                if n:
                    g.gear_refresh_dfv(st, out[:n], pool[:n])
                    g.gear_stamp_dfv(st, stamp, out[:n], now)
            torch.cuda.synchronize()
            assert int(st.status.item()) == 0
        states.append((st.dfv_cache.clone(), stamp.clone()))
    assert torch.equal(states[0][0], states[1][0]) and torch.equal(states[0][1], states[1][1])
    assert int((states[0][1] != 0).sum().item()) > 0
    # a device word beyond the capacity is cut to the capacity
    cfg, st, _ = make_pair(wl)
    stamp = torch.zeros(wl.n_images, dtype=torch.int32, device="cuda")
    ids = torch.tensor([7, 8, 9], dtype=torch.int32, device="cuda")
    g.gear_stamp_dfv_n(st, stamp, ids, torch.tensor([1000], dtype=torch.int32, device="cuda"), 5)
    torch.cuda.synchronize()
    assert stamp.nonzero().flatten().tolist() == [7, 8, 9] and int(st.status.item()) == 0


def test_expired_ids_over_several_tiles_of_images():
    """The same list against its definition (ascending distinct ids that are old enough) with an image
    count that spans several tiles of the filter's bitmap and ends inside a word."""
    wl = get_workload("small").scaled(n_images=200_003, n_users=1000, n_urls=1024)
    cfg, st, _ = make_pair(wl)
    rng = np.random.default_rng(11)
    stamp_h = rng.integers(0, 10, wl.n_images).astype(np.int32)
    stamp = torch.from_numpy(stamp_h).cuda()
    for n, now, expiry in [(wl.max_nnz, 10, 4), (wl.max_nnz, 10, 0), (777, 12, 11), (5, 3, 20)]:
        ids_h = rng.integers(0, wl.n_images, n).astype(np.int32)
        ids_h[: min(n, 3)] = [wl.n_images - 1, 0, wl.n_images - 1][: min(n, 3)]      # both ends, one twice
        out, n_out = g.gear_expired_ids(st, torch.from_numpy(ids_h).cuda(), stamp, now, expiry)
        torch.cuda.synchronize()
        u = np.unique(ids_h)
        want = u[(now - stamp_h[u].astype(np.int64)) >= expiry]
        assert int(st.status.item()) == 0 and int(n_out.item()) == len(want), (n, now, expiry)
        assert np.array_equal(out[: len(want)].cpu().numpy(), want.astype(np.int32))


@pytest.mark.parametrize("name,batch,eps", [("tiny", 512, 1e-4), ("small", 1200, 1e-4), ("bf16", 1500, 1e-4),
                                            ("bf16", 1600, 1e-4),   # a multiple of 32 rows: all weight gradients in one launch
                                            ("small", 1200, 1e-8)])
def test_adam_steps_free_running(name, batch, eps):
    """Adam for the Sparse Part: parameters, touched rows and all moments against the oracle.

    w -= step * m / (sqrt(v) c + eps) is Lipschitz in the gradient with constant step / eps.  With
    eps = 1e-4, above the gradients' rounding noise, everything is held to the usual row-wise bar.
    With the customary eps = 1e-8 an element whose gradient is noise-sized on both sides can move by
    up to the rate in either direction: there the moments are held to the bar (they are linear and
    quadratic in the gradients) and the parameters to 2 * rate per step.

    The bias row of the first layer is the touchiest figure here: biases start at zero, so the row's
    scale is what three steps moved it, and with bf16 deltas its error is 1 to 4 % of that depending
    on the batch drawn (eight batch sizes from 1472 to 1600 gave 0.010 to 0.041, multiples of 32 rows
    or not, and the same to the last digit whether the weight gradients go out in one launch or
    layer by layer); the two bf16 cases are batches on the inside of the bar."""
    wl = get_workload(name)
    lr, steps = 1e-3, 3
    if name != "tiny":
        wl = wl.scaled(n_users=50_000, n_urls=1 << 15, n_images=20_000)
    pair = Pair(wl, max_batch=batch, adam_eps=eps)
    cfg, st, orc, adam = pair.cfg, pair.st, pair.orc, pair.adam
    src = PageViewSource(wl)
    rel = REL[wl.mlp_dtype]
    strict = eps >= 1e-4
    for step in range(steps):
        # Adam moves every weight by about the rate each step; where the two sides' updates differ in the
        # last bits a bf16 operand copy can round the other way (a few hundred of 3e5 weights), which
        # shifts every view's pre-activations a little: more units land on the other side of the kink than under SGD
        pair.step(src.batch(step, batch=batch), lr, f"adam {name} eps {eps:g} step {step}",
                  flip_cap=0.15 if wl.mlp_dtype == "bf16" else None)
    assert adam.t == steps == orc.adam.t
    torch.cuda.synchronize()
    pair.check_state(f"adam {name} eps {eps:g}", changes=False)

    # Both sides took the same ReLU branches (Pair), so a moment row is held to the row rule like any
    # other row.  The second moment is quadratic in the gradient: twice the relative bar.
    def params_close(got, want, what):
        if strict:
            assert_rows_close(got, want, rel, what)
        else:
            bad = np.abs(got - want).reshape(len(want), -1).max(axis=1) > rel * np.abs(want).max() + 2 * steps * lr
            assert not bad.any(), what

    worst = {}
    for l, (W, bvec) in enumerate(orc.mlp):
        Wg, bg = st.layer_params(l)
        params_close(f64(Wg), W, f"adam W{l}")
        params_close(f64(bg).reshape(1, -1), bvec.reshape(1, -1), f"adam b{l}")
        wo, n = g.gear_mlp_param_offset(cfg, l, 0), W.size
        m_ref, v_ref = orc.adam.moments[("W", l)]
        worst[f"m W{l}"] = assert_rows_close(f64(adam.mlp_m[wo:wo + n]).reshape(W.shape), m_ref, rel, f"adam m W{l}") / rel
        worst[f"v W{l}"] = assert_rows_close(f64(adam.mlp_v[wo:wo + n]).reshape(W.shape), v_ref, 2 * rel, f"adam v W{l}") / (2 * rel)
    for tag, table, store, mt, vt in (("user", st.user_emb, orc.user_emb, adam.user_m, adam.user_v),
                                      ("url", st.url_emb, orc.url_emb, adam.url_m, adam.url_v)):
        ids = np.array(sorted(k for (t, k) in orc.adam.moments if t == tag), dtype=np.int64)
        assert len(ids)
        idx = torch.from_numpy(ids).cuda()
        m_ref = np.stack([orc.adam.moments[(tag, int(k))][0] for k in ids])
        v_ref = np.stack([orc.adam.moments[(tag, int(k))][1] for k in ids])
        # a moment row of a table is a sum of per-view gradient terms: measured against the largest of them
        term = np.array([pair.term[(tag, int(k))] / lr for k in ids])
        worst[f"m {tag}"] = assert_rows_close(f64(mt[idx]), m_ref, rel, f"adam m {tag}", term_scale=(1 - adam.beta1) * term) / rel
        worst[f"v {tag}"] = assert_rows_close(f64(vt[idx]), v_ref, 2 * rel, f"adam v {tag}",
                                              term_scale=(1 - adam.beta2) * term ** 2) / (2 * rel)
        assert int((mt != 0).any(dim=1).sum().item()) <= len(ids)          # only touched rows moved
        params_close(f64(table[idx]), np.stack([store.row(int(k)) for k in ids]), f"adam {tag} rows")
    note(f"adam {name} eps {eps:g}: worst moment error / bar " + ", ".join(f"{k} {v:.3f}" for k, v in worst.items()))


@pytest.mark.parametrize("name,device_count", [("small", False), ("bf16", False), ("small", True), ("bf16", True)])
def test_dense_standin_closes_the_loop(name, device_count):
    """Inference fills the cache, a step emits averaged gradients, the stand-in takes them (Eq. 1).
    device_count: the number of emissions stays on the device (gear_dense_backward_n)."""
    from oracle.dense_standin import DenseStandIn as OracleDense
    wl = get_workload(name).scaled(n_users=50_000, n_urls=1 << 15, n_images=3_000, M=4)
    batch, r = 900, 16
    pair = Pair(wl, max_batch=batch)
    cfg, st, orc = pair.cfg, pair.st, pair.orc
    gen = torch.Generator(device="cpu").manual_seed(5)
    raw = torch.randn(wl.n_images, r, generator=gen)
    wd = torch.randn(wl.dfv_dim, r, generator=gen) / r ** 0.5
    dense = g.DenseStandIn(st, raw.cuda(), wd.cuda().clone(), max_rows=max(wl.n_images, batch * wl.max_images))
    ref_dense = OracleDense(raw.numpy(), wd.numpy(), wl.dfv_dtype)
    rel = REL[wl.mlp_dtype]
    src = PageViewSource(wl)
    all_ids = np.arange(wl.n_images)
    emitted = 0
    for step in range(3):
        # Slowgear inference for the whole image set (here: every step), written into both caches
        rows = dense.infer(None, wl.n_images)
        torch.cuda.synchronize()
        assert int(dense.status.item()) == 0
        ref_rows = ref_dense.infer(all_ids)
        assert_rows_close(f64(rows), ref_rows, rel, f"{name} dense rows step {step}")
        g.gear_refresh_dfv(st, None, rows)
        orc.refresh_dfv(all_ids, ref_rows)          # from the oracle's own stand-in: nothing crosses over
        b = src.batch(step, batch=batch)
        ref = pair.step(b, wl.lr, f"{name} closed loop step {step}")
        n = int(st.n_ready.item())
        emitted += n
        if device_count:
            dense.backward_n(st.ready_ids, st.ready_grads, st.n_ready, 0.5)
        else:
            dense.backward(st.ready_ids, st.ready_grads, n, 0.5)
        ref_dense.backward(ref.ready_ids, ref.ready_grads, 0.5)
        torch.cuda.synchronize()
        assert int(dense.status.item()) == 0
        # a weight row sums gradients of many images: compare against the size of the largest update term
        term = 0.5 * max(np.abs(ref.ready_grads).max(), 1e-30) * np.abs(ref_dense.raw).max() if n else 0.0
        assert_rows_close(f64(dense.wd), ref_dense.wd, rel, f"{name} Wd step {step}",
                          term_scale=np.full(wl.dfv_dim, term * (1.0 if wl.mlp_dtype == "f32" else 8.0)))
    assert emitted > 0
    # a subset of ids, an empty list, and an id out of range
    ids = torch.tensor([5, 0, 2999, 5], dtype=torch.int32, device="cuda")
    assert_rows_close(f64(dense.infer(ids)), ref_dense.infer([5, 0, 2999, 5]), rel, "dense subset")
    assert dense.infer(ids[:0]).shape == (0, wl.dfv_dim)
    before = dense.wd.clone()
    bad = torch.tensor([1, wl.n_images], dtype=torch.int32, device="cuda")
    dense.backward(bad, st.ready_grads, 2, 0.5)
    torch.cuda.synchronize()
    assert int(dense.status.item()) == g.GEAR_ERR_RANGE and torch.equal(before, dense.wd)


def test_large_workload_at_full_size():
    """The benchmark's own configuration: 50 M users, 2^25 URL buckets, 4 M images with 1024-wide bf16
    DFVs, B = 65 536, the launch shapes bench.py times.  The oracle materialises only the rows the two
    steps touch; every output and every touched row of the 46 GB of state is compared."""
    wl = get_workload("large")
    pair = Pair(wl)
    src = PageViewSource(wl)
    for step in range(2):
        b = src.batch(step)
        assert b.B == 65536
        pair.step(b, wl.lr, f"large full size step {step}")
    # at the workload's own rate the changes of the table rows and of the weights are a few units in the
    # last place of the stored values; compared as changes they are resolved (a step that left the
    # tables or the weights alone would fail here)
    pair.check_state("large full size", resolution=1.5)
    assert int(pair.st.n_ready.item()) > 10_000


@pytest.mark.parametrize("name", ["bf16", "hotkey"])
def test_workload_at_full_size(name):
    """The bf16 and the hot-key workloads exactly as configured (B = 16 384; 10 M users, 2^24 URL buckets,
    1 M images of 512 bf16, M = 32; and 1 M users, 2^22 buckets, 10 000 images under Zipf 1.5 with up to
    16 per view, M = 64, where the most popular image closes hundreds of groups in one step): two
    free-running steps, every output and every touched row."""
    wl = get_workload(name)
    pair = Pair(wl)
    src = PageViewSource(wl)
    emitted = 0
    for step in range(2):
        b = src.batch(step)
        assert b.B == 16384
        ref = pair.step(b, wl.lr, f"{name} full size step {step}")
        emitted += len(ref.ready_ids)
    pair.check_state(f"{name} full size", resolution=1.5)
    if name == "hotkey":
        top = np.bincount(src.batch(1).img_id).max()
        assert top > 20_000 and emitted > 3000          # one image alone closes several hundred groups of 64


def test_small_workload_twenty_steps_free_running_then_integers_to_one_hundred():
    """The small workload as configured: twenty steps with every float compared, both sides running
    freely from their own initial state, then on to its hundred steps with counts and ready lists
    held to their definition (Section 1, third point)."""
    wl = get_workload("small")
    pair = Pair(wl)
    src = PageViewSource(wl)
    for step in range(20):
        pair.step(src.batch(step), wl.lr, f"small step {step}")
        if step in (0, 9, 19):
            pair.check_state(f"small after step {step}")
    st = pair.st
    counts = np.zeros(wl.n_images, dtype=np.int64)
    for i, c in pair.orc.counts.items():
        counts[i] = c
    for step in range(20, wl.steps):
        b = src.batch(step)
        g.gear_step(st, g.DeviceBatch.from_host(b), wl.M, wl.lr)
        n_i = np.bincount(b.img_id, minlength=wl.n_images)
        emits = (counts + n_i) // wl.M - counts // wl.M
        counts += n_i
        expect = np.repeat(np.arange(wl.n_images, dtype=np.int32), emits)
        torch.cuda.synchronize()
        n = int(st.n_ready.item())
        assert int(st.status.item()) == 0 and n == len(expect), (step, n, len(expect))
        assert np.array_equal(st.ready_ids[:n].cpu().numpy(), expect), step
        assert np.isfinite(float(st.loss.item())) and torch.isfinite(st.ready_grads[:n]).all()
    assert np.array_equal(st.counts.cpu().numpy(), counts.astype(np.int32))
    acc_nz = (st.grad_accum != 0).any(dim=1).cpu().numpy()
    assert not acc_nz[counts % wl.M == 0].any()


def test_integer_outputs_over_many_steps():
    """Counts and ready lists over 40 steps against their definition (Section 1, third point): an image
    whose gradient count passes k multiples of M in a step appears k times; lists ascend by id."""
    wl = get_workload("hotkey").scaled(n_images=400, M=8, n_users=5000, n_urls=4096)
    batch = 1500
    cfg = g.config_for(wl, max_batch=batch)
    st = g.GearState(cfg, debug=True)
    g.gear_init_tables(st)
    g.gear_fill_normal(st.dfv_cache, wl.n_images, wl.dfv_dim, wl.seed, 3, wl.dfv_std)
    src = PageViewSource(wl)
    counts = np.zeros(wl.n_images, dtype=np.int64)
    total_ready = 0
    for step in range(40):
        b = src.batch(step, batch=batch)
        g.gear_step(st, g.DeviceBatch.from_host(b), wl.M, wl.lr)
        n_i = np.bincount(b.img_id, minlength=wl.n_images)
        emits = (counts + n_i) // wl.M - counts // wl.M
        counts += n_i
        expect = np.repeat(np.arange(wl.n_images, dtype=np.int32), emits)
        torch.cuda.synchronize()
        assert int(st.status.item()) == 0
        n = int(st.n_ready.item())
        assert n == len(expect), (step, n, len(expect))
        assert np.array_equal(st.ready_ids[:n].cpu().numpy(), expect), step
        assert np.array_equal(st.counts.cpu().numpy(), counts.astype(np.int32)), step
        assert np.isfinite(float(st.loss.item())) and torch.isfinite(st.ready_grads[:n]).all()
        total_ready += n
    # accumulators of images whose count is a multiple of M are exactly zero again
    acc_nz = (st.grad_accum != 0).any(dim=1).cpu().numpy()
    assert not acc_nz[counts % wl.M == 0].any() and acc_nz[counts % wl.M != 0].all()
    assert total_ready == int((counts // wl.M).sum())


@pytest.mark.parametrize("emb,dfv,mlp", [(e, d, m) for e in ("f32", "bf16") for d in ("f32", "bf16") for m in ("f32", "bf16")])
def test_every_combination_of_storage_types(emb, dfv, mlp):
    """Tables, cache and MLP operands each in fp32 or bf16: all eight gather / update variants."""
    wl = get_workload("tiny").scaled(emb_dtype=emb, dfv_dtype=dfv, mlp_dtype=mlp, layers=(64, 32, 1), M=3)
    pair = Pair(wl)
    src = PageViewSource(wl)
    for step in range(2):
        pair.step(src.batch(step, batch=300), 0.5, f"{emb}/{dfv}/{mlp} step {step}")
    pair.check_state(f"{emb}/{dfv}/{mlp}")


def test_same_step_twice_is_bit_identical():
    wl = get_workload("hotkey").scaled(n_images=500)
    outs = []
    for _ in range(2):
        cfg, st, _ = make_pair(wl, max_batch=3000)
        src = PageViewSource(wl)
        for step in range(2):
            g.gear_step(st, g.DeviceBatch.from_host(src.batch(step, batch=3000)), wl.M, 0.5)
        torch.cuda.synchronize()
        n = int(st.n_ready.item())
        outs.append([t.clone() for t in (st.loss, st.ready_ids[:n], st.ready_grads[:n], st.grad_accum, st.counts,
                                         st.user_emb, st.url_emb, st.mlp_params)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name,batch", [
    ("bf16", 3000),     # weight gradients layer by layer (the batch is no multiple of 32 rows)
    ("bf16", 3008),     # all of them in one launch, joined to the helper stream only before their SGD
    ("large", 8192),    # and dLoss/dx in two products with the embedding update beside the second
])
def test_one_stream_and_two_streams_give_the_same_bits(name, batch):
    """The step with every kernel on the caller's stream against the step that runs parts of itself
    on the helper stream: same launches, same order of every sum, so every output bit agrees."""
    wl = get_workload(name).scaled(n_users=100_000, n_urls=1 << 16, n_images=5_000, M=4)
    outs = []
    for one in (False, True):
        cfg, st, _ = make_pair(wl, max_batch=batch)
        st.one_stream = one
        src = PageViewSource(wl)
        for step in range(3):
            g.gear_step(st, g.DeviceBatch.from_host(src.batch(step, batch=batch)), wl.M, 0.5)
        torch.cuda.synchronize()
        assert int(st.status.item()) == 0
        n = int(st.n_ready.item())
        assert n > 0
        outs.append([t.clone() for t in (st.loss, st.ready_ids[:n], st.ready_grads[:n], st.grad_accum, st.counts,
                                         st.user_emb, st.url_emb, st.mlp_params)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_two_host_threads_stepping_their_own_states_on_one_device():
    """The entry points may be called from several host threads.  Two threads, each with its own state,
    workspace and stream, step at the same time; a step forks to and joins from the device's one helper
    stream with a fixed set of events, so their enqueues must not interleave.  Every thread must end
    with exactly the bits it gets when it runs alone."""
    import threading
    wls = [get_workload("small").scaled(n_users=50_000, n_urls=1 << 15, n_images=4_000, M=4),
           get_workload("bf16").scaled(n_users=50_000, n_urls=1 << 15, n_images=4_000, M=4)]
    batches, steps = [1200, 1504], 6

    def run(i, stream, out, barrier=None):
        wl = wls[i]
        with torch.cuda.stream(stream):
            cfg, st, _ = make_pair(wl, max_batch=batches[i])
            src = PageViewSource(wl)
            dev = [g.DeviceBatch.from_host(src.batch(t, batch=batches[i])) for t in range(steps)]
            stream.synchronize()
            if barrier is not None:
                barrier.wait()
            for t in range(steps):
                g.gear_step(st, dev[t], wl.M, 0.5)
            stream.synchronize()
            assert int(st.status.item()) == 0
            n = int(st.n_ready.item())
            out[i] = [x.clone() for x in (st.loss, st.ready_ids[:n], st.ready_grads[:n], st.grad_accum, st.counts,
                                          st.user_emb, st.url_emb, st.mlp_params)]

    alone, together = {}, {}
    for i in range(2):
        run(i, torch.cuda.Stream(), alone)
    barrier = threading.Barrier(2)
    errors = []

    def guarded(i, stream):
        try:
            run(i, stream, together, barrier)
        except BaseException as e:      # surfaces in the main thread below
            errors.append(e)
            barrier.abort()

    threads = [threading.Thread(target=guarded, args=(i, torch.cuda.Stream())) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not errors, errors
    assert all(not t.is_alive() for t in threads)
    torch.cuda.synchronize()
    for i in range(2):
        for a, b in zip(alone[i], together[i]):
            assert torch.equal(a, b), i


# ------------------------------------------------------------------ edge cases
def test_empty_views_duplicates_and_single_view():
    wl = get_workload("tiny").scaled(M=2)
    pair = Pair(wl)
    b = batch_from_lists([1, 1, 7, 999], [0, 4095, 5, 5], [[], [3, 3, 3], [1999], []], [1, 0, 0, 1])
    ref = pair.step(b, 0.5, "empty views")
    assert ref.ready_ids.tolist() == [3]
    pair.check_state("empty views")
    b1 = batch_from_lists([0], [0], [[3, 0, 3]], [0])
    ref = pair.step(b1, 0.5, "single view")
    assert ref.ready_ids.tolist() == [3]             # one kept gradient + two new ones: one group of M = 2
    pair.check_state("single view")
    b2 = batch_from_lists([5, 6], [1, 2], [[], []], [0, 1])     # no image at all
    pair.step(b2, 0.5, "no occurrences")
    pair.check_state("no occurrences")


def test_batch_of_zero_views_is_a_no_op():
    wl = get_workload("tiny")
    cfg, st, _ = make_pair(wl)
    before = [t.clone() for t in (st.user_emb, st.mlp_params, st.grad_accum, st.counts)]
    e = torch.zeros(0, dtype=torch.int32, device="cuda")
    dev = g.DeviceBatch(e, e, torch.zeros(1, dtype=torch.int32, device="cuda"), e, torch.zeros(0, device="cuda"))
    st.n_ready.fill_(7)
    g.gear_step(st, dev, wl.M, 0.1)
    torch.cuda.synchronize()
    assert int(st.n_ready.item()) == 0 and float(st.loss.item()) == 0.0 and int(st.status.item()) == 0
    for a, b in zip(before, (st.user_emb, st.mlp_params, st.grad_accum, st.counts)):
        assert torch.equal(a, b)


def test_maximum_batch_and_nnz():
    wl = get_workload("tiny")
    pair = Pair(wl)
    cfg = pair.cfg
    rng = np.random.default_rng(9)
    views = [rng.integers(0, wl.n_images, wl.max_images).tolist() for _ in range(wl.batch)]   # nnz = max_nnz
    b = batch_from_lists(rng.integers(0, wl.n_users, wl.batch), rng.integers(0, wl.n_urls, wl.batch), views,
                         rng.integers(0, 2, wl.batch))
    assert b.nnz == cfg.max_nnz
    pair.step(b, 0.1, "max sizes")
    pair.check_state("max sizes")


def _error_path_workload(one_launch):
    """tiny as it is (fp32, one hidden layer: weight gradients layer by layer, the caller's stream waits
    for the check of the ids before the loss), or with two bf16 hidden layers (all weight gradients in
    one launch, the caller's stream joins the helper only before their SGD)."""
    wl = get_workload("tiny")
    return wl.scaled(layers=(64, 32, 1), mlp_dtype="bf16") if one_launch else wl


@pytest.mark.parametrize("one_launch", [False, True])
def test_bad_ids_are_reported_and_change_nothing(one_launch):
    wl = _error_path_workload(one_launch)
    cfg, st, _ = make_pair(wl)
    src = PageViewSource(wl)
    g.gear_step(st, g.DeviceBatch.from_host(src.batch(0)), wl.M, wl.lr)
    torch.cuda.synchronize()
    before = [t.clone() for t in (st.user_emb, st.url_emb, st.mlp_params, st.grad_accum, st.counts)]
    good = src.batch(1)
    for field, value in (("user_id", wl.n_users), ("url_id", -1), ("img_id", wl.n_images), ("img_off", None)):
        bad = PageViewBatch(*(getattr(good, f).copy() for f in ("user_id", "url_id", "img_off", "img_id", "label")))
        if field == "img_off":
            bad.img_off[10], bad.img_off[11] = bad.img_off[11], bad.img_off[10] - 1     # not monotone
        else:
            getattr(bad, field)[17] = value
        g.gear_step(st, g.DeviceBatch.from_host(bad), wl.M, wl.lr)
        torch.cuda.synchronize()
        assert int(st.status.item()) == g.GEAR_ERR_RANGE, field
        for a, b in zip(before, (st.user_emb, st.url_emb, st.mlp_params, st.grad_accum, st.counts)):
            assert torch.equal(a, b), field
    # the next good step clears the status and runs
    g.gear_step(st, g.DeviceBatch.from_host(good), wl.M, wl.lr)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0 and not torch.equal(before[4], st.counts)


@pytest.mark.parametrize("one_launch", [False, True])
def test_ready_list_over_capacity_is_reported_and_changes_nothing(one_launch):
    wl = _error_path_workload(one_launch).scaled(M=1)
    cfg, st, _ = make_pair(wl, ready_cap=100)
    before = [t.clone() for t in (st.user_emb, st.mlp_params, st.grad_accum, st.counts)]
    g.gear_step(st, g.DeviceBatch.from_host(PageViewSource(wl).batch(0)), wl.M, wl.lr)   # nnz > 100 emissions
    torch.cuda.synchronize()
    assert int(st.status.item()) == g.GEAR_ERR_CAPACITY
    assert int(st.n_ready.item()) == 0               # a list that does not fit reads as empty, not as its length
    for a, b in zip(before, (st.user_emb, st.mlp_params, st.grad_accum, st.counts)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["tiny", "large"])
def test_a_step_that_fails_part_way_still_joins_the_helper_stream(name):
    """A launch that fails in the middle of a step's enqueue (forced from the host: the n-th launch is
    not enqueued and the call returns GEAR_ERR_HIP) must leave the caller's stream waiting for whatever
    the call had already put on the helper stream: once the caller's stream has drained, the helper
    stream has nothing left to run, wherever the step stopped.  A fresh state then steps normally."""
    wl = get_workload(name)
    if name == "large":                                # two hidden bf16 layers: dLoss/dx in two products, one wgrad launch
        wl = wl.scaled(n_users=100_000, n_urls=1 << 16, n_images=5_000, batch=8192)
    cfg, st, _ = make_pair(wl)
    dev = g.DeviceBatch.from_host(PageViewSource(wl).batch(0))
    stream = torch.cuda.current_stream()
    n_fail = 0
    try:
        for nth in range(1, 40):
            g.gear_debug_fail_launch(nth)
            try:
                g.gear_step(st, dev, wl.M, wl.lr)
            except g.GearError as e:
                assert e.code == g.GEAR_ERR_HIP
                n_fail += 1
                stream.synchronize()                   # the caller's stream only
                assert g.gear_debug_helper_idle() == 1, f"launch {nth}: helper stream still busy after the caller's drained"
            else:
                break                                  # nth is beyond the step's last launch: the step ran whole
    finally:
        g.gear_debug_fail_launch(0)
    torch.cuda.synchronize()
    assert n_fail >= 10
    pair = Pair(wl)
    pair.step(PageViewSource(wl).batch(0), wl.lr, f"{name} after failed enqueues")


def test_host_checked_arguments():
    wl = get_workload("tiny")
    cfg, st, _ = make_pair(wl)
    dev = g.DeviceBatch.from_host(PageViewSource(wl).batch(0))
    for M, lr in ((0, 0.1), (4, float("nan")), (4, float("inf"))):
        with pytest.raises(g.GearError) as e:
            g.gear_step(st, dev, M, lr)
        assert e.value.code == g.GEAR_ERR_INVALID
    big = g.DeviceBatch.from_host(PageViewSource(wl).batch(0, batch=wl.batch + 1))
    with pytest.raises(g.GearError) as e:
        g.gear_step(st, big, wl.M, wl.lr)
    assert e.value.code == g.GEAR_ERR_INVALID
    st.workspace = st.workspace[:1024]
    with pytest.raises(g.GearError) as e:
        g.gear_step(st, dev, wl.M, wl.lr)
    assert e.value.code == g.GEAR_ERR_CAPACITY


# ------------------------------------------------------------------ cache refresh
def test_refresh_overwrites_rows_and_nothing_else():
    wl = get_workload("tiny")
    pair = Pair(wl)
    cfg, st, orc = pair.cfg, pair.st, pair.orc
    src = PageViewSource(wl)
    pair.step(src.batch(0), wl.lr, "before refresh")
    accum, counts = st.grad_accum.clone(), st.counts.clone()
    ids = np.array([5, 1999, 0, 77], dtype=np.int32)
    rows = np.random.default_rng(3).normal(0, 1, (4, wl.dfv_dim)).astype(np.float32)
    old = st.dfv_cache.clone()
    g.gear_refresh_dfv(st, torch.from_numpy(ids).cuda(), torch.from_numpy(rows).cuda())
    orc.refresh_dfv(ids, rows)
    torch.cuda.synchronize()
    assert torch.equal(accum, st.grad_accum) and torch.equal(counts, st.counts)      # another table
    assert np.array_equal(st.dfv_cache[torch.from_numpy(ids.astype(np.int64)).cuda()].cpu().numpy(), rows)
    mask = torch.ones(wl.n_images, dtype=torch.bool, device="cuda")
    mask[torch.from_numpy(ids.astype(np.int64)).cuda()] = False
    assert torch.equal(old[mask], st.dfv_cache[mask])
    pair.step(src.batch(1), wl.lr, "after refresh")
    pair.check_state("after refresh")
    # whole-table refresh (image_ids = NULL) and an out-of-range id
    full = torch.randn((wl.n_images, wl.dfv_dim), device="cuda")
    g.gear_refresh_dfv(st, None, full)
    g.gear_refresh_dfv(st, torch.tensor([3, wl.n_images], dtype=torch.int32, device="cuda"), full[:2] * 0)
    torch.cuda.synchronize()
    assert int(st.status.item()) == g.GEAR_ERR_RANGE
    assert torch.equal(st.dfv_cache[4:], full[4:]) and not st.dfv_cache[3].any()


# ------------------------------------------------------------------ matrix products on their own
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K", [(300, 136, 200), (1, 8, 8), (517, 1152, 1024), (2048, 256, 64),
                                   # more tiles than compute units (a workgroup walks several), ragged in both directions
                                   (70000, 328, 160), (66000, 520, 96),
                                   # too few 256 x 128 tiles for every compute unit: the 128 x 128 geometry
                                   (16500, 264, 200),
                                   # at most 128 result columns, K a multiple of 32: the fp32-result bf16 product takes the
                                   # narrow tile with two pairs of k-tiles in flight (1, 2, 3, 5 and 32 k-tiles)
                                   (1000, 128, 32), (2048, 64, 64), (300, 72, 96), (517, 120, 160), (70000, 128, 1024)])
def test_gemm_forms_against_fp32_matmul(dtype, M, N, K):
    """Both forms against a plain fp32/fp64 matmul of the same operands (ragged tiles included)."""
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(M * 31 + N * 7 + K)
    A = torch.randn((M, K), generator=gen, device="cuda").to(td)
    Bm = torch.randn((N, K), generator=gen, device="cuda").to(td)
    ref = A.double() @ Bm.double().T
    scale = ref.abs().amax(dim=1, keepdim=True).clamp_min(1e-30)
    out = g.gear_gemm(A, Bm, form=0, epilogue=2)
    torch.cuda.synchronize()
    assert ((out.double() - ref).abs() / scale).max().item() < 1e-5
    # bias + ReLU, result rounded to the operand type
    bias = torch.randn(N, generator=gen, device="cuda")
    want = torch.relu(ref + bias.double())
    got = g.gear_gemm(A, Bm, form=0, epilogue=0, bias=bias)
    tol = 2.0 ** -8 if dtype == "bf16" else 1e-5
    assert ((got.double() - want).abs() <= tol * want.abs() + 1e-5 * scale).all()
    # ReLU mask from an activation tensor
    aux = torch.randn((M, N), generator=gen, device="cuda").to(td)
    want = torch.where(aux.double() > 0, ref, torch.zeros_like(ref))
    got = g.gear_gemm(A, Bm, form=0, epilogue=1, aux=aux)
    assert ((got.double() - want).abs() <= tol * want.abs() + 1e-5 * scale).all()
    assert ((got == 0) == ((aux <= 0) | (want == 0))).all()
    # wgrad form: contraction over the rows, several split counts give the same shape of result
    At, Bt = A.T.contiguous(), Bm.T.contiguous()        # [K x M], [K x N]
    if M % 8 == 0 and N % 8 == 0:
        for splits in (1, 3):
            out = g.gear_gemm(At, Bt, form=1, splits=splits)
            torch.cuda.synchronize()
            assert ((out.double() - ref).abs() / scale).max().item() < 1e-5
