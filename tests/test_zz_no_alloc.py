"""gear_step_static (the step on the library's static scratch array, for callers that cannot allocate)
against gear_step with a caller's workspace: the same kernels in the same order, so every output and
every piece of state must agree bit for bit.  Two calls in a row, the second with a smaller batch, so
that whatever the first call left in the shared array is met by the second."""
import numpy as np
import pytest
import torch

from gear_inputs import PageViewSource, get_workload

pytestmark = pytest.mark.gpu


def _state(g, wl, max_batch):
    st = g.GearState(g.config_for(wl, max_batch=max_batch), debug=True)
    g.gear_init_tables(st)
    g.gear_fill_normal(st.dfv_cache, wl.n_images, wl.dfv_dim, wl.seed, 3, wl.dfv_std)
    return st


def _outputs(st):
    n, nu = int(st.n_ready.item()), int(st.dbg[3].item())
    return [t.clone() for t in (st.loss, st.n_ready, st.status, st.ready_ids[:n], st.ready_grads[:n], st.grad_accum,
                                st.counts, st.user_emb, st.url_emb, st.mlp_params, st.dbg[0][:nu], st.dbg[1][:nu + 1],
                                st.dbg[3])]


@pytest.mark.parametrize("name", ["small", "bf16"])
def test_step_on_static_scratch_matches_step_on_a_workspace(name):
    import paper_1806_03925_amd as g
    assert torch.cuda.is_available(), "this test needs the GPU"
    wl = get_workload(name).scaled(n_users=100_000, n_urls=1 << 16, n_images=5_000, M=4)
    first, second = (4096, 1000) if name == "small" else (3008, 777)
    assert g.gear_workspace_bytes(g.config_for(wl, max_batch=first)) <= 64 << 20
    src = PageViewSource(wl)
    ref, dut = _state(g, wl, first), _state(g, wl, first)
    dut.workspace = None                                   # the static variant must not need it
    for step, batch in enumerate((first, second)):
        b = g.DeviceBatch.from_host(src.batch(step, batch=batch))
        print(f"static scratch: {name} step {step} B {batch}", flush=True)
        g.gear_step(ref, b, wl.M, 0.5)
        g.gear_step_static(dut, b, wl.M, 0.5)
        torch.cuda.synchronize()
        assert int(ref.status.item()) == 0 and int(dut.status.item()) == 0
        assert int(ref.n_ready.item()) > 0
        for a, c in zip(_outputs(ref), _outputs(dut)):
            assert torch.equal(a, c), (name, step)
    assert not np.array_equal(ref.counts.cpu().numpy(), np.zeros(wl.n_images, np.int32))


def test_static_scratch_rejects_a_configuration_that_does_not_fit():
    import paper_1806_03925_amd as g
    wl = get_workload("hotkey")                             # 107 MiB of workspace at B = 16 384
    st = g.GearState(g.config_for(wl.scaled(n_users=1000, n_urls=1024, n_images=1000)))
    g.gear_init_tables(st)
    before = [t.clone() for t in (st.user_emb, st.mlp_params, st.grad_accum, st.counts)]
    b = g.DeviceBatch.from_host(PageViewSource(wl.scaled(n_users=1000, n_urls=1024, n_images=1000)).batch(0, batch=64))
    with pytest.raises(g.GearError) as e:
        g.gear_step_static(st, b, wl.M, 0.1)
    assert e.value.code == g.GEAR_ERR_CAPACITY
    torch.cuda.synchronize()
    for a, c in zip(before, (st.user_emb, st.mlp_params, st.grad_accum, st.counts)):
        assert torch.equal(a, c)


def test_static_step_replays_from_a_graph():
    """The step on the static scratch array launches everything on one stream and allocates nothing, so
    a caller can record it into a graph.  A graph fixes the batch's shape (B and the number of
    occurrences are launch arguments), so the workload here has one image per view; the batch's
    contents change between replays through the same device buffers.  Each replay, with eager work and
    synchronisations in between, must leave exactly what the eager step leaves."""
    import paper_1806_03925_amd as g
    wl = get_workload("epoch").scaled(batch=600, n_images=1800, M=2)
    src = PageViewSource(wl)

    def state():
        st = g.GearState(g.config_for(wl), debug=False)
        g.gear_init_tables(st)
        g.gear_fill_normal(st.dfv_cache, wl.n_images, wl.dfv_dim, wl.seed, 3, wl.dfv_std)
        return st

    ref, dut = state(), state()
    first = g.DeviceBatch.from_host(src.batch(0))
    slot = g.DeviceBatch(*(t.clone() for t in (first.user_id, first.url_id, first.img_off, first.img_id, first.label)))
    torch.cuda.synchronize()
    # warm-up outside the graph on a scratch state (first-use set-up must not happen under capture)
    g.gear_step_static(state(), slot, wl.M, wl.lr)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g.gear_step_static(dut, slot, wl.M, wl.lr)
    torch.cuda.synchronize()
    before = [t.clone() for t in (dut.counts, dut.grad_accum, dut.user_emb, dut.mlp_params)]
    for a, b in zip(before, (ref.counts, ref.grad_accum, ref.user_emb, ref.mlp_params)):
        assert torch.equal(a, b)                        # recording ran nothing
    for step in range(5):
        b = g.DeviceBatch.from_host(src.batch(step))
        assert b.nnz == slot.nnz and b.B == slot.B
        for dst, s in zip((slot.user_id, slot.url_id, slot.img_off, slot.img_id, slot.label),
                          (b.user_id, b.url_id, b.img_off, b.img_id, b.label)):
            dst.copy_(s)
        graph.replay()
        g.gear_step(ref, b, wl.M, wl.lr)
        torch.cuda.synchronize()
        n = int(ref.n_ready.item())
        assert int(dut.status.item()) == 0 and int(dut.n_ready.item()) == n, step
        for a, c in zip((ref.loss, ref.ready_ids[:n], ref.ready_grads[:n], ref.grad_accum, ref.counts, ref.user_emb,
                         ref.url_emb, ref.mlp_params),
                        (dut.loss, dut.ready_ids[:n], dut.ready_grads[:n], dut.grad_accum, dut.counts, dut.user_emb,
                         dut.url_emb, dut.mlp_params)):
            assert torch.equal(a, c), step
    assert int(ref.counts.sum().item()) == 5 * 600
