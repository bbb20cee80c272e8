"""sp_greedy_round_static (the entry point that allocates nothing: its round kernels exchange their
candidates through the library's static device array) against sp_greedy_round, through the C ABI.

Two windows in a row on the same GPU, the second smaller in every dimension (fewer applications,
variants, batch sizes and requests), so that the static array still holds the first window's words
when the second one runs.  Both entry points start from identically scored contexts; every round's
decision record, status and member ids must be bit-identical, and so must the schedule that follows.
"""
import numpy as np
import pytest

from paper_2505_06641_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    from paper_2505_06641_amd import binding
    binding.load_library()
    return torch, binding


def rounds_both_ways(gpu, w, n_rounds):
    """n_rounds single-round calls on two contexts of the same window: one through each entry point."""
    torch, binding = gpu
    p, rq = w.profile, w.requests
    x, app, D, wt = binding.to_device(rq)
    B = int(p.max_batch)
    got = {}
    for name in ("sp_greedy_round", "sp_greedy_round_static"):
        ctx = binding.Context(p, rq.n)
        ctx.sp_score(x, app, D, wt)
        ids = torch.full((B,), -1, dtype=torch.int32, device="cuda:0")
        recs = []
        for _ in range(n_rounds):
            ids.fill_(-1)
            rc, d = getattr(ctx, name)(req_ids_out=ids)
            recs.append((rc, d, ids.cpu().numpy().copy()))
            if rc != binding.SP_OK:
                break
        # the rest of the window on the ordinary path: the state the single rounds left must be the same
        n = rq.n
        model = torch.full((n,), 99, dtype=torch.int32, device="cuda:0")
        order = torch.full((n,), 99, dtype=torch.int32, device="cuda:0")
        util = torch.full((n,), -7.0, device="cuda:0")
        rc, summ, log = ctx.sp_schedule(16, model, None, order, util, log_capacity=n)
        got[name] = (recs, rc, summ, log, model.cpu().numpy(), order.cpu().numpy(), util.cpu().numpy())
        ctx.close()
    return got["sp_greedy_round"], got["sp_greedy_round_static"]


def assert_same(ref, new):
    recs_a, rc_a, summ_a, log_a, model_a, order_a, util_a = ref
    recs_b, rc_b, summ_b, log_b, model_b, order_b, util_b = new
    assert len(recs_a) == len(recs_b) and len(recs_a) > 0
    for (ra, da, ia), (rb, db, ib) in zip(recs_a, recs_b):
        assert ra == rb
        assert da == db                      # every field of the decision record, bit for bit
        assert np.array_equal(ia, ib)
    assert rc_a == rc_b and summ_a == summ_b and log_a == log_b
    assert np.array_equal(model_a, model_b) and np.array_equal(order_a, order_b)
    assert np.array_equal(util_a.view(np.uint32), util_b.view(np.uint32))


def test_static_round_matches_twice_in_a_row_second_window_smaller(gpu):
    big = wl.make("cfg4", n_requests=8192)       # 8 applications, 8 variants, batch sizes up to 64
    small = wl.make("cfg2", n_requests=700)      # 3 applications, 4 variants, batch sizes up to 32
    ref, new = rounds_both_ways(gpu, big, 12)
    assert any(r[1] is not None and r[1]["batch"] > 1 for r in ref[0])
    assert_same(ref, new)
    ref, new = rounds_both_ways(gpu, small, 12)
    assert_same(ref, new)


def test_static_round_status_codes(gpu):
    torch, binding = gpu
    w = wl.tiny(seed=5, n=6)
    ctx = binding.Context(w.profile, 16)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_greedy_round_static()
    assert e.value.status == binding.SP_ESTATE          # before the first sp_score
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    seen = 0
    while True:
        rc, d = ctx.sp_greedy_round_static()
        if rc == binding.SP_DONE:
            break
        seen += d["batch"]
        assert seen <= 6
    rc, d = ctx.sp_greedy_round_static()                 # after the end: still SP_DONE
    assert rc == binding.SP_DONE and d is None
    ctx.close()


def test_static_round_rejects_what_does_not_fit(gpu):
    torch, binding = gpu
    # 2,100 applications x 128 batch sizes: the window-position table alone is over 1 MiB
    w = wl.tiny(seed=6, n=32, classes=(2,) * 2100, models=(1,) * 2100, max_batch=128)
    ctx = binding.Context(w.profile, 64)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_greedy_round_static()
    assert e.value.status == binding.SP_ECAPACITY
    rc, d = ctx.sp_greedy_round()                        # the context is still usable
    assert rc == binding.SP_OK
    ctx.close()
