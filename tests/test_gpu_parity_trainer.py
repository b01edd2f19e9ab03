"""GPU parity of Alg. 1 end to end (WARMUP passes, then FormalTraining) through
cdsgd_trainer_step, against the oracle's trainer, every iteration, on ragged layer lists.
Both sources of the 32-bit aggregate are covered: summed in the kernel from the N gradients
(cdsgd_plan_bind_full_grads) and read from agg_full."""
import numpy as np
import pytest
import torch

from helpers import assert_bits_equal, assert_close

pytestmark = pytest.mark.gpu

SIZES = [4096, 4097, 1000, 64, 10, 36864, 20011, 1]


@pytest.fixture(scope="module")
def P():
    import paper_2106_10796_amd as pkg
    from paper_2106_10796_amd import build, runner, synth
    build.ensure_built()
    pkg.binding.lib()
    assert torch.cuda.is_available()
    return pkg, runner, synth


@pytest.mark.parametrize("full_grads", [True, False], ids=["kernel_sum", "agg_full"])
@pytest.mark.parametrize("warmup_n,N,self_rank,k,base", [
    (0, 4, 0, 3, "c2_resnet20"), (1, 8, 5, 4, "c2_resnet20"), (3, 16, 15, 2, "c3_resnet50"),
    (2, 1, 0, 3, "c1_single"), (2, 3, 1, 1, "c5_flat4g"), (0, 5, 3, 2, "c5_flat4g"), (0, 1, 0, 2, "c1_single")])
def test_trainer_matches_oracle(P, oracle, full_grads, warmup_n, N, self_rank, k, base):
    pkg, runner, synth = P
    cfg = synth.scaled(synth.config(base), SIZES, "_trainer")
    cfg.num_workers, cfg.k = N, k
    wl = runner.Workload(cfg, dense=True, self_rank=self_rank, full_grads=full_grads)
    lr_l, lr_g = 0.4, 0.1
    trainer = pkg.Trainer(wl.plan, warmup_n, k, cfg.threshold, lr_l, lr_g)
    blocks = [(i, 0, n) for i, n in enumerate(cfg.sizes)]
    # the local buffer starts at a sentinel unrelated to the weights, on both sides: Alg. 1 writes it
    # before it ever reads it (for warmup_n = 0 the base of pass 0's local update is the global weight)
    SENTINEL = -1234.5
    wl.w_local.fill_(SENTINEL)
    sims = [oracle.TrainerSimulation(wl.view(wl.w_global, i).cpu().numpy(), N, warmup_n, k, cfg.threshold,
                                     lr_l, lr_g, self_rank, w_local0=np.full(cfg.sizes[i], SENTINEL, np.float32))
            for i in range(cfg.num_tensors)]
    kinds = []
    for it in range(warmup_n + 1 + 2 * k + 1):
        count = it - warmup_n - 1
        comp = it > warmup_n and count % k != 0
        cap = wl.prepare_step(it, capture=blocks, compressed=comp)
        loc_before = wl.w_local.clone()
        res_before = wl.residual.clone()
        assert trainer.iteration == it
        kind = trainer.step()
        torch.cuda.synchronize()
        kinds.append(kind)
        for i in range(cfg.num_tensors):
            mode, agg, words = sims[i].step([cap[j][i] for j in range(N)])
            assert mode == kind
            tag = "iteration %d tensor %d (n=%d)" % (it, i, cfg.sizes[i])
            if mode == 1:
                assert_bits_equal(wl.pview(wl.packed_self, i).cpu().numpy(), words[self_rank].view(np.int32),
                                  "packed " + tag)
            else:
                assert torch.equal(wl.view(wl.residual, i), wl.view(res_before, i)), "residual touched " + tag
            assert_bits_equal(wl.view(wl.residual, i).cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
            gw, gl = wl.view(wl.w_global, i).cpu().numpy(), wl.view(wl.w_local, i).cpu().numpy()
            assert_close(gw, sims[i].w_global, "w_global " + tag)
            assert_close(gl, sims[i].w_local, "w_local " + tag)
            assert_bits_equal(gw, sims[i].w_global, "w_global bits " + tag)
            assert_bits_equal(gl, sims[i].w_local, "w_local bits " + tag)
            if mode == 0 and it < warmup_n - 1:
                assert torch.equal(wl.view(wl.w_local, i), wl.view(loc_before, i)), "w_local written early " + tag
                assert bool((wl.view(wl.w_local, i) == SENTINEL).all()), "w_local written early " + tag
    expect = [0] * (warmup_n + 1) + [2 if c % k == 0 else 1 for c in range(2 * k + 1)]
    assert kinds == expect
    trainer.destroy()
    wl.destroy()


def test_full_pass_needs_an_aggregate(P):
    """A plan with neither agg_full nor bound gradients cannot run a correction or warm-up pass."""
    pkg, runner, synth = P
    B = pkg.binding
    n = 100
    mk = lambda: torch.zeros(n, device="cuda")
    t = dict(w_global=mk(), w_local=mk(), residual=mk(), grad=mk(), packed_self=B.new_packed(n))
    plan = B.Plan([t], [None, [B.new_packed(n)]], 2, 0)
    with pytest.raises(B.CdsgdError) as e:
        plan.step(0, 4, 0.5, 0.1, 0.1)
    assert e.value.status == B.ERR_NULL
    with pytest.raises(B.CdsgdError) as e:
        plan.step_warmup(0, 2, 0.1, 0.1)
    assert e.value.status == B.ERR_NULL
    plan.step(1, 4, 0.5, 0.1, 0.1)      # compressed passes do not need it
    torch.cuda.synchronize()
    plan.destroy()


@pytest.mark.parametrize("max_workgroups", [0, 1, 5, 64], ids=["wg_per_chunk", "1wg", "5wg", "64wg"])
@pytest.mark.parametrize("t_pow2", [True, False], ids=["t0.5", "t0.05"])
def test_split_step_equals_fused(P, oracle, t_pow2, max_workgroups):
    """cdsgd_step_local then cdsgd_step_global (on a second stream, ordered by an event)
    leave bit for bit what cdsgd_step_fused leaves, on compressed and correction passes;
    cdsgd_step_local alone matches eq. 11 of the oracle and leaves w_global alone.  The split
    side also runs with a bounded number of workgroups (cdsgd_plan_set_max_workgroups): fewer
    workgroups than chunks, each walking several, must change nothing."""
    pkg, runner, synth = P
    cfg = synth.scaled(synth.config("c2_resnet20" if t_pow2 else "c5_flat4g"), SIZES, "_split")
    cfg.num_workers, cfg.k = 8, 3
    a = runner.Workload(cfg, dense=True, self_rank=3)     # fused
    b = runner.Workload(cfg, dense=True, self_rank=3)     # split
    b.plan.set_max_workgroups(max_workgroups)
    side = torch.cuda.Stream()                            # default priority
    main = torch.cuda.current_stream()
    for s in range(2 * cfg.k + 1):
        a.prepare_step(s)
        b.prepare_step(s)
        a.fused_step(s)
        wg_before = b.w_global.clone()
        b.plan.step_local(cfg.lr)
        local_done = torch.cuda.Event()
        local_done.record(main)
        torch.cuda.synchronize()
        # eq. 11 alone, against the oracle
        for i in range(cfg.num_tensors):
            W = b.view(wg_before, i).cpu().numpy()
            L = np.zeros_like(W)
            oracle.update(W, L, b.view(b.grad, i).cpu().numpy(), None, cfg.lr, cfg.lr, cfg.num_workers)
            assert_bits_equal(b.view(b.w_local, i).cpu().numpy(), L, "w_local after step_local, step %d tensor %d" % (s, i))
        assert torch.equal(b.w_global, wg_before)
        with torch.cuda.stream(side):
            side.wait_event(local_done)
            b.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr)
        torch.cuda.synchronize()
        for key in ("w_global", "w_local", "residual", "packed_self"):
            x, y = getattr(a, key), getattr(b, key)
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), "%s differs at step %d" % (key, s)
    a.destroy()
    b.destroy()


@pytest.mark.parametrize("full_grads", [True, False], ids=["kernel_sum", "agg_full"])
def test_workgroup_limit_changes_nothing(P, oracle, full_grads):
    """Alg. 1 end to end (warm-up, correction and compressed passes) on a plan limited to 1, 2, 7
    or far more workgroups than it has chunks, against the same plan without a limit: every
    buffer bit for bit, every iteration; the unlimited run is itself checked against the oracle
    by the other tests of this file."""
    pkg, runner, synth = P
    cfg = synth.scaled(synth.config("c5_flat4g"), SIZES + [3 * 4096 + 17], "_wglimit")
    cfg.num_workers, cfg.k = 5, 3
    warmup_n = 1
    limits = [0, 1, 2, 7, 1 << 20]
    wls = [runner.Workload(cfg, dense=True, self_rank=2, full_grads=full_grads) for _ in limits]
    trainers = []
    for wl, lim in zip(wls, limits):
        wl.plan.set_max_workgroups(lim)
        trainers.append(pkg.Trainer(wl.plan, warmup_n, cfg.k, cfg.threshold, 0.4, 0.1))
    for it in range(warmup_n + 1 + 2 * cfg.k):
        comp = it > warmup_n and (it - warmup_n - 1) % cfg.k != 0
        for wl, tr in zip(wls, trainers):
            wl.prepare_step(it, compressed=comp)
            tr.step()
        torch.cuda.synchronize()
        for wl, lim in zip(wls[1:], limits[1:]):
            for key in ("w_global", "w_local", "residual", "packed_self"):
                x, y = getattr(wls[0], key), getattr(wl, key)
                assert torch.equal(x.view(torch.int32), y.view(torch.int32)), \
                    "%s differs at iteration %d with a limit of %d workgroups" % (key, it, lim)
    with pytest.raises(pkg.CdsgdError) as e:
        wls[0].plan.set_max_workgroups(-1)
    assert e.value.status == pkg.binding.ERR_PARAM
    for tr in trainers:
        tr.destroy()
    for wl in wls:
        wl.destroy()


@pytest.mark.parametrize("by_ranges", [False, True], ids=["whole_list", "layer_ranges"])
def test_fused_steps_in_a_hip_graph_replay_like_eager(P, by_ranges):
    """The step is launch-bound on small layer lists, so a caller may capture a run of steps
    in a HIP graph.  The library enqueues kernels only (no memset or copy nodes), so a captured
    period of k steps must replay, several times and with eager work in between, to exactly
    the state the eager calls reach.  by_ranges: the graph holds every step as five launches over
    ranges of layers, last layers first; the eager side still steps the whole list."""
    pkg, runner, synth = P
    cfg = synth.config("c2_resnet20")
    a = runner.Workload(cfg, dense=True)     # eager
    b = runner.Workload(cfg, dense=True)     # graph
    for wl in (a, b):
        wl.prepare_step(0)                   # agg_full for the correction step of the period
        wl.prepare_step(1)                   # own gradient and the peers' packed streams
    period = list(range(cfg.k))              # one correction step + k-1 compressed steps

    def run_period(wl):
        for s in period:
            if by_ranges and wl is b:
                for lo, hi in ((60, 65), (41, 60), (40, 41), (7, 40), (0, 7)):
                    wl.plan.step_range(lo, hi - lo, s, cfg.k, cfg.threshold, cfg.lr, cfg.lr)
            else:
                wl.fused_step(s)

    assert cfg.num_tensors == 65
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):            # warm-up on the capture stream, as torch asks
        run_period(b)
    torch.cuda.current_stream().wait_stream(side)
    run_period(a)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_period(b)
    for rep in range(4):
        graph.replay()
        run_period(a)
        torch.cuda.synchronize()
        # eager work between the replays, touching other memory
        junk = torch.randn(1 << 20, device="cuda").sum().item()
        assert junk == junk
        for key in ("w_global", "w_local", "residual", "packed_self"):
            x, y = getattr(a, key), getattr(b, key)
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), "%s differs after replay %d" % (key, rep)
    a.destroy()
    b.destroy()


@pytest.mark.parametrize("full_grads", [True, False], ids=["kernel_sum", "agg_full"])
@pytest.mark.parametrize("dtype", ["bfloat16", "float16"])
def test_low_precision_gradients(P, oracle, dtype, full_grads):
    """Gradients held in bf16 / fp16 (cdsgd_plan_create_typed): every pass must give exactly
    what the fp32 oracle gives on the widened values, through warm-up, correction and
    compressed passes, for both thresholds' decode forms."""
    pkg, runner, synth = P
    gd = getattr(torch, dtype)
    for base, N, self_rank in (("c2_resnet20", 4, 1), ("c5_flat4g", 5, 4)):
        cfg = synth.scaled(synth.config(base), SIZES, "_lowp")
        cfg.num_workers, cfg.k = N, 3
        wl = runner.Workload(cfg, dense=True, self_rank=self_rank, full_grads=full_grads, grad_dtype=gd)
        lr_l, lr_g, warmup_n = 0.4, 0.1, 1
        trainer = pkg.Trainer(wl.plan, warmup_n, cfg.k, cfg.threshold, lr_l, lr_g)
        blocks = [(i, 0, n) for i, n in enumerate(cfg.sizes)]
        sims = [oracle.TrainerSimulation(wl.view(wl.w_global, i).cpu().numpy(), N, warmup_n, cfg.k, cfg.threshold,
                                         lr_l, lr_g, self_rank) for i in range(cfg.num_tensors)]
        fired = 0
        for it in range(warmup_n + 1 + 2 * cfg.k):
            count = it - warmup_n - 1
            comp = it > warmup_n and count % cfg.k != 0
            cap = wl.prepare_step(it, capture=blocks, compressed=comp)
            # what the library reads is the low-precision buffer; the oracle gets its exact widening
            own = [wl.view(wl.grad, i).float().cpu().numpy() for i in range(cfg.num_tensors)]
            kind = trainer.step()
            torch.cuda.synchronize()
            for i in range(cfg.num_tensors):
                assert np.array_equal(own[i], cap[self_rank][i])
                mode, agg, words = sims[i].step([cap[j][i] for j in range(N)])
                assert mode == kind
                tag = "%s iteration %d tensor %d" % (dtype, it, i)
                if mode == 1:
                    assert_bits_equal(wl.pview(wl.packed_self, i).cpu().numpy(), words[self_rank].view(np.int32),
                                      "packed " + tag)
                    fired += int(np.count_nonzero(words[self_rank]))
                assert_bits_equal(wl.view(wl.residual, i).cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
                assert_bits_equal(wl.view(wl.w_global, i).cpu().numpy(), sims[i].w_global, "w_global " + tag)
                assert_bits_equal(wl.view(wl.w_local, i).cpu().numpy(), sims[i].w_local, "w_local " + tag)
        assert fired > 0
        trainer.destroy()
        wl.destroy()


@pytest.mark.parametrize("pow2", [False, True], ids=["sigma", "pow2"])
def test_per_tensor_thresholds(P, oracle, pow2):
    """cdsgd_plan_set_thresholds on the literal ResNet-20 recipe (per-tensor gradient std
    log-uniform over three decades, where a single threshold of 0.5 never fires): threshold i
    = the tensor's std (chain form of the decode) or the nearest power of two (count form).
    Every tensor must fire and match its own oracle run; clearing the thresholds goes back to
    the call's threshold."""
    import math
    pkg, runner, synth = P
    cfg = synth.config("c2_resnet20")
    th = [float(np.float32(s)) for s in cfg.tensor_std]
    if pow2:
        th = [2.0 ** round(math.log2(s)) for s in th]
    wl = runner.Workload(cfg, self_rank=2)
    wl.set_thresholds(th)
    N = cfg.num_workers
    blocks = [(i, 0, n) for i, n in enumerate(cfg.sizes)]
    sims = [oracle.Simulation(wl.view(wl.w_global, i).cpu().numpy(), N, cfg.k, th[i], cfg.lr, cfg.lr, 2)
            for i in range(cfg.num_tensors)]
    fired = np.zeros(cfg.num_tensors, np.int64)
    for s in range(2 * cfg.k):
        cap = wl.prepare_step(s, capture=blocks)
        wl.fused_step(s)                      # the call's threshold (0.5) must be ignored
        torch.cuda.synchronize()
        for i in range(cfg.num_tensors):
            comp, agg, words = sims[i].step([cap[j][i] for j in range(N)])
            tag = "step %d tensor %d (t=%g)" % (s, i, th[i])
            if comp:
                assert_bits_equal(wl.pview(wl.packed_self, i).cpu().numpy(), words[2].view(np.int32), "packed " + tag)
                for j in range(N):
                    if j != 2:
                        assert_bits_equal(wl.pview(wl.peer_packed[j], i).cpu().numpy(), words[j].view(np.int32),
                                          "peer packed " + tag)
                fired[i] += int(np.count_nonzero(words[2]))
            assert_bits_equal(wl.view(wl.residual, i).cpu().numpy(), sims[i].residual[2], "residual " + tag)
            assert_bits_equal(wl.view(wl.w_global, i).cpu().numpy(), sims[i].w_global, "w_global " + tag)
            assert_bits_equal(wl.view(wl.w_local, i).cpu().numpy(), sims[i].w_local, "w_local " + tag)
    assert (fired > 0).all()                  # with its own threshold every tensor sends codes
    # back to the single threshold of the call for every tensor
    wl.set_thresholds(None)
    wl.prepare_step(1)
    r_before = wl.residual.clone()
    wl.packed_self.fill_(-1)
    wl.fused_step(1)
    torch.cuda.synchronize()
    for i in range(cfg.num_tensors):
        r = wl.view(r_before, i).cpu().numpy()
        words = oracle.quantize_pack(wl.view(wl.grad, i).cpu().numpy(), r, cfg.threshold)
        assert_bits_equal(wl.pview(wl.packed_self, i).cpu().numpy(), words.view(np.int32), "packed after clearing, tensor %d" % i)
        assert_bits_equal(wl.view(wl.residual, i).cpu().numpy(), r, "residual after clearing, tensor %d" % i)
    wl.destroy()
