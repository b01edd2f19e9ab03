"""GPU test of cdsgd_step_fused_static, the fused step for callers that cannot allocate:
through the C ABI, against cdsgd_step_fused on a plan built from the same layer list, bit for
bit (packed codes, residuals, both weights), on calls in a row that share the library's static
device array -- the second with a smaller input than the first."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

GUARD = 64


@pytest.fixture(scope="module")
def B():
    from paper_2106_10796_amd import binding, build
    build.ensure_built()
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _guarded(values, dtype, fill):
    n = len(values)
    full = torch.full((n + 2 * GUARD,), fill, dtype=dtype, device="cuda")
    full[GUARD: GUARD + n].copy_(torch.as_tensor(values, dtype=dtype))
    return full


def _make_case(B, rng, sizes, N, self_rank, t, grad_dtype):
    """Two identical device copies of a layer list's state (one per entry point) and the peers'
    streams (read-only, shared).  Every buffer sits between sentinels."""
    copies = []
    host = []
    for n in sizes:
        g = rng.normal(0, 1.1 * t, n).astype(np.float32)
        host.append(dict(
            w_global=rng.normal(0, 0.3, n).astype(np.float32),
            residual=rng.uniform(-t, t, n).astype(np.float32),
            grad=g,
            agg_full=rng.normal(0, 2.0 * t, n).astype(np.float32)))
    for _ in range(2):
        fulls, tensors = [], []
        for n, h in zip(sizes, host):
            f = dict(
                w_global=_guarded(h["w_global"], torch.float32, 5.0),
                w_local=_guarded(np.full(n, -77.0, np.float32), torch.float32, 6.0),
                residual=_guarded(h["residual"], torch.float32, 7.0),
                grad=_guarded(h["grad"], grad_dtype, 8.0),
                packed_self=torch.full((B.packed_words(n) + 2 * GUARD,), -1, dtype=torch.int32, device="cuda"),
                agg_full=_guarded(h["agg_full"], torch.float32, 9.0))
            fulls.append(f)
            tensors.append({key: (v[GUARD: GUARD + (B.packed_words(n) if key == "packed_self" else n)])
                            for key, v in f.items()})
        copies.append((fulls, tensors))
    peers = None
    if N > 1:
        peers = []
        for j in range(N):
            if j == self_rank:
                peers.append(None)
                continue
            row = []
            for n in sizes:
                codes = rng.choice(3, size=B.packed_words(n) * 16, p=[0.5, 0.3, 0.2]).astype(np.uint64)
                words = (codes.reshape(-1, 16) << (2 * np.arange(16, dtype=np.uint64))).sum(axis=1).astype(np.uint32)
                row.append(torch.from_numpy(words.view(np.int32)).cuda())
            peers.append(row)
    return copies, peers


def _assert_same(copies, tag):
    (fa, _), (fb, _) = copies
    for i, (x, y) in enumerate(zip(fa, fb)):
        for key in ("w_global", "w_local", "residual", "packed_self", "grad", "agg_full"):
            a, b = x[key], y[key]
            if a.dtype != torch.int32:
                a, b = a.view(torch.int16 if a.element_size() == 2 else torch.int32), \
                    b.view(torch.int16 if b.element_size() == 2 else torch.int32)
            assert torch.equal(a, b), "%s: %s of tensor %d differs (guards included)" % (tag, key, i)


def _run_pair(B, rng, sizes, N, self_rank, t, steps, k, grad_dtype=torch.float32, lr_l=0.4, lr_g=0.1):
    copies, peers = _make_case(B, rng, sizes, N, self_rank, t, grad_dtype)
    plan = B.Plan(copies[0][1], peers, N, self_rank, grad_dtype=grad_dtype)
    marshalled = B.StaticLayerList(copies[1][1], peers, N, grad_dtype=grad_dtype)   # the same call, arrays built once
    for turn, s in enumerate(steps):
        plan.step(s, k, t, lr_l, lr_g)
        if turn % 2:
            marshalled.step(self_rank, s, k, t, lr_l, lr_g)
        else:
            B.cdsgd_step_fused_static(copies[1][1], peers, N, self_rank, s, k, t, lr_l, lr_g, grad_dtype=grad_dtype)
        torch.cuda.synchronize()
        _assert_same(copies, "sizes=%s N=%d self=%d t=%g step %d" % (sizes[:4], N, self_rank, t, s))
    # something was actually computed: weights moved, codes were written on compressed steps
    fulls, tensors = copies[1]
    assert all(bool((tt["w_local"] != -77.0).all()) for tt in tensors)
    if any(s % k for s in steps):
        assert all(bool((tt["packed_self"] != -1).all()) for tt in tensors)   # 0xFFFFFFFF is never written
    plan.destroy()
    return copies


def test_static_step_matches_plan_step_on_calls_in_a_row(B):
    rng = np.random.default_rng(707)
    # first a larger layer list (several chunks, ragged tails, chain form of the decode) ...
    big = [1, 10, 16, 17, 64, 100, 1000, 4095, 4096, 4097, 9000, 36864, 5, 20011, 300001]
    _run_pair(B, rng, big, N=5, self_rank=2, t=0.05, steps=[1, 2, 0, 4], k=3)
    # ... then a smaller one on the same static array (fewer tensors, fewer chunks, other N, count form)
    small = [1000, 17, 4097]
    copies, peers = _make_case(B, rng, small, 3, 0, 0.5, torch.float32)
    plan = B.Plan(copies[0][1], peers, 3, 0)
    for s in (1, 0, 5):
        plan.step(s, 4, 0.5, 0.4, 0.1)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        B.cdsgd_step_fused_static(copies[1][1], peers, 3, 0, s, 4, 0.5, 0.4, 0.1)
        torch.cuda.synchronize()
        # the call took no device memory (nothing else ran between the two readings)
        assert torch.cuda.mem_get_info()[0] == free_before
        _assert_same(copies, "smaller input, step %d" % s)
    plan.destroy()
    # and once more larger again, one worker only, then 16-bit gradients
    _run_pair(B, rng, [8192, 3, 70001], N=1, self_rank=0, t=0.25, steps=[0, 1], k=2)
    _run_pair(B, rng, [4100, 33, 12289], N=16, self_rank=9, t=0.3, steps=[1, 3], k=2, grad_dtype=torch.bfloat16)
    _run_pair(B, rng, [77], N=2, self_rank=1, t=0.5, steps=[1, 2], k=3, grad_dtype=torch.float16)


def test_static_steps_replay_from_a_hip_graph(B):
    """What the entry point is for: it enqueues kernels only (the tables travel in kernel arguments), so a
    period of steps can be captured in a HIP graph and replayed.  Replays, with eager work in between, must
    leave exactly what the same steps through a plan leave."""
    rng = np.random.default_rng(909)
    sizes, N, self_rank, k, t = [4097, 300, 12288, 5], 6, 4, 3, 0.5
    copies, peers = _make_case(B, rng, sizes, N, self_rank, t, torch.float32)
    plan = B.Plan(copies[0][1], peers, N, self_rank)
    period = list(range(k))                   # one correction pass, k - 1 compressed passes

    def run_static():
        for s in period:
            B.cdsgd_step_fused_static(copies[1][1], peers, N, self_rank, s, k, t, 0.4, 0.1)

    def run_plan():
        for s in period:
            plan.step(s, k, t, 0.4, 0.1)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):             # warm-up on the capture stream (also looks the array's address up)
        run_static()
    torch.cuda.current_stream().wait_stream(side)
    run_plan()
    torch.cuda.synchronize()
    _assert_same(copies, "before the capture")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_static()
    for rep in range(4):
        graph.replay()
        run_plan()
        torch.cuda.synchronize()
        junk = torch.randn(1 << 18, device="cuda").sum().item()     # eager work between the replays
        assert junk == junk
        _assert_same(copies, "after replay %d" % rep)
    plan.destroy()


def test_static_step_limits_and_errors(B):
    """Sizes beyond the static array's limits and missing inputs are refused before anything runs."""
    n = 64
    mk = lambda: torch.zeros(n, device="cuda")
    t = dict(w_global=mk(), w_local=mk(), residual=mk(), grad=mk(), packed_self=B.new_packed(n))
    peers = [None, [B.new_packed(n)]]
    before = {k: v.clone() for k, v in t.items()}
    with pytest.raises(B.CdsgdError) as e:        # correction pass without agg_full
        B.cdsgd_step_fused_static([t], peers, 2, 0, 0, 4, 0.5, 0.1, 0.1)
    assert e.value.status == B.ERR_NULL
    with pytest.raises(B.CdsgdError) as e:
        B.cdsgd_step_fused_static([t], peers, 2, 0, 1, 0, 0.5, 0.1, 0.1)
    assert e.value.status == B.ERR_PARAM
    many = [t] * (B.STATIC_MAX_TENSORS + 1)
    with pytest.raises(B.CdsgdError) as e:
        B.cdsgd_step_fused_static(many, [None, [peers[1][0]] * len(many)], 2, 0, 1, 4, 0.5, 0.1, 0.1)
    assert e.value.status == B.ERR_SIZE
    torch.cuda.synchronize()
    for k, v in t.items():
        assert torch.equal(v, before[k])          # nothing was enqueued on the error paths
    B.cdsgd_step_fused_static([t], peers, 2, 0, 1, 4, 0.5, 0.1, 0.1)   # a good call still works
    torch.cuda.synchronize()
