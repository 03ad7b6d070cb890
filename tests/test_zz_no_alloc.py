"""adam_mini_step_static (the entry point that allocates nothing: tables, partial sums and step
scales in a fixed array inside the library) against adam_mini_step, through the C ABI."""
import pytest

pytestmark = pytest.mark.gpu

BIG = [(300, 4096), (3, 49152), (2, 200000), (1, 524288), (5000, 1), (70, 64), (5, 264), (3, 11008), (2, 32768),
       (3, 101), (1, 9001)]
BIG_COLUMNS = [(1024, 300), (1000, 33), (260, 3)]
SMALL = [(40, 256), (2, 20001 * 5), (17, 1)]
SMALL_COLUMNS = [(264, 9)]
ONE_LAUNCH = [(300, 64), (5, 4096), (3, 16384), (1, 256, 0.0)]      # a list the generic one-launch kernel serves
HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def _pair(shapes, columns, grad_dtype, seed):
    """Two identical device states of one tensor list: [0] is stepped with adam_mini_step,
    [1] with adam_mini_step_static."""
    import gpu_harness as H
    import torch
    specs = H.make_specs(shapes) + H.make_specs(columns, strided=True)
    runs = [H.GpuRun(specs, grad_dtype) for _ in range(2)]
    torch.manual_seed(seed)
    for k, s in enumerate(specs):
        p0 = torch.randn(s.numel) * 0.02
        for run in runs:
            run.p[k].copy_(p0)
    return runs


def _new_grads(runs, seed):
    import torch
    torch.manual_seed(seed)
    for k, s in enumerate(runs[0].specs):
        g = (torch.randn(s.numel) * 1e-3).to(runs[0].g[k].dtype)
        for run in runs:
            run.g[k].copy_(g)


def _assert_same(runs, what):
    import torch
    torch.cuda.synchronize()
    a, b = runs
    for k in range(len(a.specs)):
        assert torch.equal(a.p[k], b.p[k]), "%s: param %d (%s)" % (what, k, a.specs[k].shape)
        assert torch.equal(a.m[k], b.m[k]), "%s: m %d (%s)" % (what, k, a.specs[k].shape)
    assert torch.equal(a.v, b.v), "%s: v" % what


@pytest.mark.parametrize("grad_dtype", ["bf16", "f32"])
def test_static_scratch_step_equals_the_allocating_step(grad_dtype, oracle):
    """Two calls in a row share the GPU's one array, the second on a smaller tensor list; then they
    alternate.  Every result equals adam_mini_step's bit for bit, and the oracle's to tolerance."""
    import gpu_harness as H
    import numpy as np
    import oracle as orc
    big = _pair(BIG, BIG_COLUMNS, grad_dtype, 1)
    small = _pair(SMALL, SMALL_COLUMNS, grad_dtype, 2)
    one = _pair(ONE_LAUNCH, [], grad_dtype, 3)
    specs = big[0].specs
    st = orc.OracleState([s.numel for s in specs], [s.block_numel for s in specs], [s.wd_scale for s in specs],
                         [x.cpu().numpy() for x in big[0].p], strided=[s.strided for s in specs])
    for t in range(1, 5):
        _new_grads(big, 10 + t)
        _new_grads(small, 20 + t)
        _new_grads(one, 30 + t)
        big[0].opt.step(step=t, **HP)
        small[0].opt.step(step=t, **HP)
        one[0].opt.step(step=t, **HP)
        big[1].opt.step(step=t, static=True, **HP)        # the array now holds the big list's tables and sums
        small[1].opt.step(step=t, static=True, **HP)      # ... and now the smaller list's, over their remains
        one[1].opt.step(step=t, static=True, **HP)
        _assert_same(big, "big list, step %d" % t)
        _assert_same(small, "small list, step %d" % t)
        _assert_same(one, "one-launch list, step %d" % t)
        st.step([H.grad_to_host(g) for g in big[1].g], orc.Hyper.from_f32(**HP))
    worst = H.compare(big[1], st, 5e-3 if grad_dtype == "bf16" else 1e-5, label="static")
    assert worst < 1e-5
    # same layout twice in a row with unchanged pointers: the tables are not rewritten, the sums are
    for t in range(5, 7):
        _new_grads(big, 10 + t)
        big[0].opt.step(step=t, **HP)
        big[1].opt.step(step=t, static=True, **HP)
    _assert_same(big, "big list, back-to-back static steps")
    # one layout may use both entry points in turn
    _new_grads(small, 99)
    small[0].opt.step(step=5, **HP)
    small[1].opt.step(step=5, **HP)
    _new_grads(small, 98)
    small[0].opt.step(step=6, **HP)
    small[1].opt.step(step=6, static=True, **HP)
    _assert_same(small, "small list, mixed entry points")
    for run in big + small + one:
        run.close()


def test_static_scratch_step_first_call_and_new_pointers():
    """The very first call on a fresh layout goes through the static entry point (nothing was ever
    allocated for it), and its gradient buffers move between calls."""
    import torch
    runs = _pair(SMALL + [(64, 4096)], SMALL_COLUMNS, "bf16", 3)
    for t in range(1, 4):
        torch.manual_seed(40 + t)
        fresh = [(torch.randn(s.numel) * 1e-3).to(torch.bfloat16).cuda() for s in runs[0].specs]
        for run in runs:
            run.opt.bind(run.p, fresh, run.m, run.v)
        runs[0].opt.step(step=t, **HP)
        runs[1].opt.step(step=t, static=True, **HP)
        _assert_same(runs, "step %d" % t)
    for run in runs:
        run.close()


def test_static_scratch_step_replays_from_a_hip_graph():
    """A warmed-up static step enqueues kernels only, so it can be captured; every replay equals the
    eager allocating step, with eager work and synchronisation between the replays."""
    import torch
    runs = _pair(BIG, BIG_COLUMNS, "bf16", 4)
    _new_grads(runs, 5)
    for t in (1, 2):
        runs[0].opt.step(step=t, **HP)
        runs[1].opt.step(step=t, static=True, **HP)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        runs[1].opt.step(step=3, static=True, **HP)
    for replay in range(3):
        runs[0].opt.step(step=3, **HP)
        graph.replay()
        torch.cuda.synchronize()
        x = torch.randn(1 << 20, device="cuda").sum().item()
        assert x == x
        _assert_same(runs, "replay %d" % replay)
    for run in runs:
        run.close()


def test_static_scratch_limit_is_enforced():
    """A layout whose scratch does not fit the array is refused before anything is launched."""
    import torch
    from paper_2406_16793_amd import binding as B
    # column blocks of a [4096, 2^21] matrix with 64-row tiles: 64 * 2^21 partial sums = 512 MB
    h = B.adam_mini_init_layout([(4096 * (1 << 21), 4096, 1.0, B.FLAG_STRIDED)], B.GRAD_BF16, 0)
    P = B.pointer_array([0x1000])
    with pytest.raises(B.AdamMiniError) as ei:
        B.adam_mini_step_static(h, P, P, P, 0x1000, B.HParams(1e-3, 0.9, 0.95, 1e-8, 0.1, 1), 0)
    assert ei.value.status == B.TOO_LARGE
    B.adam_mini_destroy_layout(h)
    torch.cuda.synchronize()
