"""Parity of the HIP path (through the C ABI) with the CPU oracle, on a real MI355X.

Integer results are compared bit for bit, floating point by the row rule of oracle/compare.py
(1e-5 relative for fp32 workloads, 2e-2 for bf16).  Both sides start from their own counter-based
initialiser and run freely; nothing the oracle consumes comes from the GPU.
"""
import math

import numpy as np
import pytest
import torch

from gear_inputs import PageViewSource, get_workload
from gear_inputs.pageviews import PageViewBatch, batch_from_lists
from oracle import philox_normal
from oracle.compare import REL, assert_rows_close, row_errors
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


def check_step(wl, st, orc, batch: PageViewBatch, lr: float, what: str, adam=None, flip_cap=None,
               earlier_flipped_imgs=()):
    """Run one step on both sides and compare every output; returns the oracle's result."""
    rel = REL[wl.mlp_dtype]
    dev = g.DeviceBatch.from_host(batch)
    if adam is None:
        g.gear_step(st, dev, wl.M, lr)
    else:
        g.gear_step_adam(st, dev, wl.M, lr, adam)
    torch.cuda.synchronize()
    ref = orc.step(batch, float(np.float32(lr)))
    B, d = batch.B, wl.emb_dim
    assert int(st.status.item()) == 0, what

    # grouping of the image ids
    nu = int(st.dbg[3].item())
    assert nu == len(ref.img_unique), what
    assert np.array_equal(st.dbg[0][:nu].cpu().numpy(), ref.img_unique), what
    assert np.array_equal(st.dbg[1][:nu + 1].cpu().numpy(), ref.img_segoff), what
    assert np.array_equal(st.dbg[2][:batch.nnz].cpu().numpy(), ref.img_perm), what

    # forward
    assert_rows_close(f64(st.region("x", B)), ref.x, rel, f"{what}: x")
    assert_rows_close(f64(st.region("logits", B)), ref.logits, rel, f"{what}: logits")
    assert abs(float(st.loss.item()) - ref.loss) <= rel * abs(ref.loss), (what, st.loss.item(), ref.loss)

    # dLoss/dx.  A view whose hidden pre-activation lies within rounding distance of the ReLU kink
    # may take the other branch, which moves its whole row by about 1/sqrt(active units).  In fp32
    # the two sides differ by accumulation order only (~1e-6 of the layer's scale).  With bf16
    # operands an element of x or h can round to the neighbouring bf16 value (2^-8 relative), which
    # shifts the next layer's pre-activations by about 2^-8 * |w| / sqrt(fan_in) ~ 1e-3 of their
    # scale.  Rows outside that distance must pass; inside it they may flip, but only a few do.
    tol = 1e-5 if wl.mlp_dtype == "f32" else 2e-3
    near_kink = (ref.kink_margin < tol).any(axis=1)
    dx = f64(st.region("dx", B))
    assert np.isfinite(dx).all()
    err, scale = row_errors(dx, ref.dx)
    failed = err > rel * scale
    assert not (failed & ~near_kink).any(), \
        f"{what}: dx rows off away from any kink: {np.flatnonzero(failed & ~near_kink)[:5]}"
    cap = max(2, 0.002 * B) if wl.mlp_dtype == "f32" else max(2, 0.06 * B)
    if flip_cap is not None:
        cap = max(2, flip_cap * B)
    assert failed.sum() <= cap, f"{what}: {failed.sum()} of {B} dx rows flipped at kinks ({near_kink.sum()} rows are near one)"
    assert np.median(err / scale) <= rel / 4, f"{what}: median dx row error {np.median(err / scale):.2e}"
    # downstream sums inherit a view's error: views at more than half the bar (far above the rounding
    # noise of a view with no flipped unit) are treated like the failed ones when rows are exempted
    flipped_views = np.flatnonzero(err > 0.5 * rel * scale)
    flipped_imgs = set()
    for b in flipped_views:
        flipped_imgs.update(batch.img_id[batch.img_off[b]:batch.img_off[b + 1]].tolist())

    # ready list and averaged gradients
    n_ready = int(st.n_ready.item())
    assert n_ready == len(ref.ready_ids), what
    assert np.array_equal(st.ready_ids[:n_ready].cpu().numpy(), ref.ready_ids), what
    if n_ready:
        # an average can also hold gradients that flipped views of earlier steps left in the accumulator
        ex = np.isin(ref.ready_ids, list(flipped_imgs | set(earlier_flipped_imgs)))
        assert_rows_close(f64(st.ready_grads[:n_ready]), ref.ready_grads, rel, f"{what}: ready_grads", exempt=ex,
                          term_scale=ref.ready_term_scale)
    return ref, flipped_views, flipped_imgs


def check_state(wl, st, orc, what, flipped_users=(), flipped_urls=(), flipped_imgs=()):
    """Compare the persistent state: counters bit-exact, accumulators and tables by rows."""
    rel = REL[wl.mlp_dtype]
    counts = st.counts.cpu().numpy()
    touched = np.array(sorted(orc.counts), dtype=np.int64)
    assert int(counts.sum()) == sum(orc.counts.values()), what
    assert np.array_equal(counts[touched], np.array([orc.counts[i] for i in touched], dtype=np.int32)), what
    if len(touched):
        acc = f64(st.grad_accum[torch.from_numpy(touched).cuda()])
        ref = np.stack([orc.residual(i) for i in touched])
        # images whose count is a multiple of M hold exactly zero
        full = np.array([orc.counts[i] % wl.M == 0 for i in touched])
        assert not acc[full].any(), what
        assert_rows_close(acc, ref, rel, f"{what}: grad_accum", exempt=np.isin(touched, list(flipped_imgs)),
                          term_scale=[orc.residual_term_scale(i) for i in touched])
    # untouched accumulators are still zero
    nz_rows = int((st.grad_accum != 0).any(dim=1).sum().item())
    assert nz_rows <= len(touched), what
    for name, table, store, flipped in (("user_emb", st.user_emb, orc.user_emb, flipped_users),
                                        ("url_emb", st.url_emb, orc.url_emb, flipped_urls)):
        ids = np.array(sorted(store._rows), dtype=np.int64)
        if len(ids):
            got = f64(table[torch.from_numpy(ids).cuda()])
            assert_rows_close(got, np.stack([store.row(i) for i in ids]), rel, f"{what}: {name}",
                              exempt=np.isin(ids, list(flipped)))
    for l, (W, b) in enumerate(orc.mlp):
        Wg, bg = st.layer_params(l)
        assert_rows_close(f64(Wg), W, rel, f"{what}: W{l}")
        assert_rows_close(f64(bg), b, rel, f"{what}: b{l}")


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
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    emitted = 0
    for step in range(wl.steps):
        ref, fv, fi = check_step(wl, st, orc, src.batch(step), wl.lr, f"tiny step {step}")
        assert len(fv) == 0
        emitted += len(ref.ready_ids)
        check_state(wl, st, orc, f"tiny after step {step}")
    assert emitted > 0


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
    cfg, st, orc = make_pair(wl, max_batch=batch)
    src = PageViewSource(wl)
    fu, fl, fi = set(), set(), set()
    for step in range(steps):
        b = src.batch(step, batch=batch)
        ref, fv, imgs = check_step(wl, st, orc, b, lr, f"{name} B={batch} step {step}", earlier_flipped_imgs=fi)
        fu.update(b.user_id[fv].tolist()); fl.update(b.url_id[fv].tolist()); fi.update(imgs)
        check_state(wl, st, orc, f"{name} B={batch} after step {step}", fu, fl, fi)
    assert sum(orc.counts.values()) > 0


@pytest.mark.parametrize("dtype,hidden", [
    ("f32", (64, 512)),      # last hidden width 512 fp32: 128 16-byte pieces per row, two per lane
    ("f32", (32, 1024)),     # 1024 fp32: four pieces per lane (the widest the logit layer takes)
    ("bf16", (64, 1024)),    # 1024 bf16: two pieces per lane
    ("bf16", (64, 8)),       # a single piece: most lanes of a group idle
])
def test_wide_and_narrow_last_hidden_layer(dtype, hidden):
    """The logit/loss kernel picks lanes per view and pieces per lane from the last hidden width."""
    wl = get_workload("tiny").scaled(layers=(*hidden, 1), mlp_dtype=dtype, emb_dtype=dtype, dfv_dtype=dtype)
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    for step in range(2):
        b = src.batch(step, batch=389)
        check_step(wl, st, orc, b, 0.05, f"{dtype} hidden {hidden} step {step}")
    check_state(wl, st, orc, f"{dtype} hidden {hidden}")


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
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    fu, fl, fi = set(), set(), set()
    for step in range(2):
        b = src.batch(step, batch=batch)
        ref, fv, imgs = check_step(wl, st, orc, b, 0.5, f"three hidden layers B={batch} step {step}",
                                   earlier_flipped_imgs=fi)
        fu.update(b.user_id[fv].tolist()); fl.update(b.url_id[fv].tolist()); fi.update(imgs)
    check_state(wl, st, orc, f"three hidden layers B={batch}", fu, fl, fi)


def test_batches_smaller_than_the_largest_take_whichever_weight_gradient_path_fits():
    """A state sized for 1500 views (no multiple of 32 rows) steps through batches of 1472 (all weight
    gradients in one launch, more split-K partials than a layer-by-layer step of 1500 needs), 1500 and 700."""
    wl = get_workload("bf16").scaled(n_users=50_000, n_urls=1 << 15, n_images=5_000, M=4)
    cfg, st, orc = make_pair(wl, max_batch=1500)
    src = PageViewSource(wl)
    fu, fl, fi = set(), set(), set()
    for step, batch in enumerate((1472, 1500, 700)):
        b = src.batch(step, batch=batch)
        ref, fv, imgs = check_step(wl, st, orc, b, 0.05, f"max 1500, B={batch}", earlier_flipped_imgs=fi)
        fu.update(b.user_id[fv].tolist()); fl.update(b.url_id[fv].tolist()); fi.update(imgs)
    check_state(wl, st, orc, "max 1500", fu, fl, fi)


def test_epoch_pattern_free_running():
    """One image per view, every image once per epoch: cold rows each step, groups close after M epochs."""
    wl = get_workload("epoch").scaled(batch=600, n_images=1800, M=2)
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    emitted = []
    for step in range(8):                                   # 2 2/3 epochs of three steps
        ref, _, _ = check_step(wl, st, orc, src.batch(step), wl.lr, f"epoch step {step}")
        emitted.append(len(ref.ready_ids))
    check_state(wl, st, orc, "epoch after 8 steps")
    assert emitted == [0, 0, 0, 600, 600, 600, 0, 0]


def test_expired_ids_and_stamps_match_oracle():
    """Expiry of cached inference results: bit-exact lists over several steps of refresh + stamp."""
    wl = get_workload("hotkey").scaled(n_images=3000, batch=700)
    cfg, st, orc = make_pair(wl)
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
    check_step(wl, st, orc, src.batch(20), wl.lr, "step after refreshes")
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
    cfg, st, orc = make_pair(wl, max_batch=batch)
    orc.use_adam(eps=eps)
    adam = g.AdamMoments(st, eps=eps)
    src = PageViewSource(wl)
    rel = REL[wl.mlp_dtype]
    strict = eps >= 1e-4
    fu, fl, fi = set(), set(), set()
    for step in range(steps):
        b = src.batch(step, batch=batch)
        # Adam moves every weight by about the rate each step; where the two sides' updates differ in the
        # last bits a bf16 operand copy can round the other way (a few hundred of 3e5 weights), which
        # shifts every view's pre-activations a little: more units flip than under SGD
        ref, fv, imgs = check_step(wl, st, orc, b, lr, f"adam {name} step {step}", adam=adam,
                                   flip_cap=0.15 if wl.mlp_dtype == "bf16" else None)
        fu.update(b.user_id[fv].tolist()); fl.update(b.url_id[fv].tolist()); fi.update(imgs)
    assert adam.t == steps == orc.adam.t
    torch.cuda.synchronize()

    def moments_close(got, want, tol, what, exempt=None):
        # a moment row is a gradient row: in bf16 a unit that takes the other ReLU branch for one view
        # moves its whole row by about 1/sqrt(views), so there most rows must pass and none may be far off
        if wl.mlp_dtype != "bf16":
            return assert_rows_close(got, want, tol, what, exempt=exempt)
        err, scale = row_errors(got, want)
        off = err > tol * scale
        if exempt is not None:
            off &= ~exempt
        assert off.mean() <= 0.10 and (err[off] <= 0.3 * scale[off]).all(), (what, int(off.sum()), len(off))

    def params_close(got, want, what, exempt=None):
        if strict:
            assert_rows_close(got, want, rel, what, exempt=exempt)
        else:
            bad = np.abs(got - want).reshape(len(want), -1).max(axis=1) > rel * np.abs(want).max() + 2 * steps * lr
            assert not (bad & ~(np.zeros(len(bad), bool) if exempt is None else exempt)).any(), what

    for l, (W, bvec) in enumerate(orc.mlp):
        Wg, bg = st.layer_params(l)
        params_close(f64(Wg), W, f"adam W{l}")
        params_close(f64(bg).reshape(1, -1), bvec.reshape(1, -1), f"adam b{l}")
        wo, n = g.gear_mlp_param_offset(cfg, l, 0), W.size
        m_ref, v_ref = orc.adam.moments[("W", l)]
        moments_close(f64(adam.mlp_m[wo:wo + n]).reshape(W.shape), m_ref, rel, f"adam m W{l}")
        moments_close(f64(adam.mlp_v[wo:wo + n]).reshape(W.shape), v_ref, 2 * rel, f"adam v W{l}")
    for tag, table, store, mt, vt, flipped in (("user", st.user_emb, orc.user_emb, adam.user_m, adam.user_v, fu),
                                               ("url", st.url_emb, orc.url_emb, adam.url_m, adam.url_v, fl)):
        ids = np.array(sorted(k for (t, k) in orc.adam.moments if t == tag), dtype=np.int64)
        assert len(ids)
        idx = torch.from_numpy(ids).cuda()
        ex = np.isin(ids, list(flipped))
        m_ref = np.stack([orc.adam.moments[(tag, int(k))][0] for k in ids])
        v_ref = np.stack([orc.adam.moments[(tag, int(k))][1] for k in ids])
        moments_close(f64(mt[idx]), m_ref, rel, f"adam m {tag}", exempt=ex)
        moments_close(f64(vt[idx]), v_ref, 2 * rel, f"adam v {tag}", exempt=ex)
        assert int((mt != 0).any(dim=1).sum().item()) <= len(ids)          # only touched rows moved
        params_close(f64(table[idx]), np.stack([store.row(int(k)) for k in ids]), f"adam {tag} rows", exempt=ex)


@pytest.mark.parametrize("name,device_count", [("small", False), ("bf16", False), ("small", True), ("bf16", True)])
def test_dense_standin_closes_the_loop(name, device_count):
    """Inference fills the cache, a step emits averaged gradients, the stand-in takes them (Eq. 1).
    device_count: the number of emissions stays on the device (gear_dense_backward_n)."""
    from oracle.dense_standin import DenseStandIn as OracleDense
    wl = get_workload(name).scaled(n_users=50_000, n_urls=1 << 15, n_images=3_000, M=4)
    batch, r = 900, 16
    cfg, st, orc = make_pair(wl, max_batch=batch)
    gen = torch.Generator(device="cpu").manual_seed(5)
    raw = torch.randn(wl.n_images, r, generator=gen)
    wd = torch.randn(wl.dfv_dim, r, generator=gen) / r ** 0.5
    dense = g.DenseStandIn(st, raw.cuda(), wd.cuda().clone(), max_rows=max(wl.n_images, batch * wl.max_images))
    ref_dense = OracleDense(raw.numpy(), wd.numpy(), wl.dfv_dtype)
    rel = REL[wl.mlp_dtype]
    src = PageViewSource(wl)
    all_ids = np.arange(wl.n_images)
    emitted, fi = 0, set()
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
        ref, fv, imgs = check_step(wl, st, orc, b, wl.lr, f"{name} closed loop step {step}", earlier_flipped_imgs=fi)
        fi.update(imgs)
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
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    fu, fl, fi = set(), set(), set()
    for step in range(2):
        b = src.batch(step)
        assert b.B == 65536
        ref, fv, imgs = check_step(wl, st, orc, b, wl.lr, f"large full size step {step}", earlier_flipped_imgs=fi)
        fu.update(b.user_id[fv].tolist()); fl.update(b.url_id[fv].tolist()); fi.update(imgs)
    check_state(wl, st, orc, "large full size", fu, fl, fi)
    assert int(st.n_ready.item()) > 10_000


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
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    fu, fl, fi = set(), set(), set()
    for step in range(2):
        b = src.batch(step, batch=300)
        ref, fv, imgs = check_step(wl, st, orc, b, 0.5, f"{emb}/{dfv}/{mlp} step {step}", earlier_flipped_imgs=fi)
        fu.update(b.user_id[fv].tolist()); fl.update(b.url_id[fv].tolist()); fi.update(imgs)
    check_state(wl, st, orc, f"{emb}/{dfv}/{mlp}", fu, fl, fi)


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


# ------------------------------------------------------------------ edge cases
def test_empty_views_duplicates_and_single_view():
    wl = get_workload("tiny").scaled(M=2)
    cfg, st, orc = make_pair(wl)
    b = batch_from_lists([1, 1, 7, 999], [0, 4095, 5, 5], [[], [3, 3, 3], [1999], []], [1, 0, 0, 1])
    ref, _, _ = check_step(wl, st, orc, b, 0.5, "empty views")
    assert ref.ready_ids.tolist() == [3]
    check_state(wl, st, orc, "empty views")
    b1 = batch_from_lists([0], [0], [[3, 0, 3]], [0])
    ref, _, _ = check_step(wl, st, orc, b1, 0.5, "single view")
    assert ref.ready_ids.tolist() == [3]             # one kept gradient + two new ones: one group of M = 2
    check_state(wl, st, orc, "single view")
    b2 = batch_from_lists([5, 6], [1, 2], [[], []], [0, 1])     # no image at all
    check_step(wl, st, orc, b2, 0.5, "no occurrences")
    check_state(wl, st, orc, "no occurrences")


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
    cfg, st, orc = make_pair(wl)
    rng = np.random.default_rng(9)
    views = [rng.integers(0, wl.n_images, wl.max_images).tolist() for _ in range(wl.batch)]   # nnz = max_nnz
    b = batch_from_lists(rng.integers(0, wl.n_users, wl.batch), rng.integers(0, wl.n_urls, wl.batch), views,
                         rng.integers(0, 2, wl.batch))
    assert b.nnz == cfg.max_nnz
    check_step(wl, st, orc, b, 0.1, "max sizes")
    check_state(wl, st, orc, "max sizes")


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
    for a, b in zip(before, (st.user_emb, st.mlp_params, st.grad_accum, st.counts)):
        assert torch.equal(a, b)


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
    cfg, st, orc = make_pair(wl)
    src = PageViewSource(wl)
    check_step(wl, st, orc, src.batch(0), wl.lr, "before refresh")
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
    check_step(wl, st, orc, src.batch(1), wl.lr, "after refresh")
    check_state(wl, st, orc, "after refresh")
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
                                   (70000, 328, 160), (66000, 520, 96)])
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
