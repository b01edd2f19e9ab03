"""GPU parity on the five workloads, in the launch configuration the benchmark times.

Small workloads (single tensor, ResNet-20-shaped list) are compared whole, every step,
fused and three-call path, literal and dense value recipes.  The large ones (ResNet-50,
VGG-16, 4 GiB flat bucket) run at full size and are compared on sampled blocks that the
oracle can recompute one by one (first / last / ragged-tail / random blocks; the path is
elementwise, so a block of outputs depends only on the same block of inputs), plus, over
the whole buffers, fused == three-call path bit for bit and the conservation property of
the quantiser.  The two layer lists are also compared element by element, whole, for three
iterations, and the 4 GiB bucket for its first two.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from helpers import assert_bits_equal, assert_close, count_bit_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2106_10796_amd as pkg
    from paper_2106_10796_amd import build, runner, synth
    build.ensure_built()
    pkg.binding.lib()
    assert torch.cuda.is_available()
    return pkg, runner, synth


def _whole(cfg):
    return [(i, 0, n) for i, n in enumerate(cfg.sizes)]


def _sample_blocks(cfg, rng, nblocks, blen):
    """(tensor, start, length): starts are multiples of 16; blocks either end on a multiple
    of 16 or at the tensor's (possibly ragged) end."""
    out = []
    order = np.argsort(cfg.sizes)[::-1]
    big = int(order[0])
    n = cfg.sizes[big]
    out.append((big, 0, min(blen, n)))                                   # first block
    out.append((big, max(0, (n - blen) // 16 * 16), n - max(0, (n - blen) // 16 * 16)))  # last block
    ragged = [i for i, m in enumerate(cfg.sizes) if m % 16]
    for i in ragged[:4]:                                                 # ragged tails
        m = cfg.sizes[i]
        s = max(0, (m - 2048) // 16 * 16)
        out.append((i, s, m - s))
    small = [i for i in order[::-1][:3]]                                 # smallest tensors, whole
    for i in small:
        out.append((int(i), 0, min(cfg.sizes[i], blen)))
    while len(out) < nblocks:
        i = int(rng.choice(len(cfg.sizes), p=np.array(cfg.sizes) / sum(cfg.sizes)))
        m = cfg.sizes[i]
        ln = min(blen, m)
        s = int(rng.integers(0, (m - ln) // 16 + 1)) * 16
        out.append((i, s, min(ln, m - s)))
    return out


def _partition(cfg, blen):
    """Every element of every tensor, in blocks of at most blen elements (blen a multiple of 16)."""
    assert blen % 16 == 0
    return [(i, a, min(blen, n - a)) for i, n in enumerate(cfg.sizes) for a in range(0, n, blen)]


def _run(P, oracle, cfg, dense, steps, blocks, fused=True, self_rank=0, check_peers=True, shadow=False,
         wl_kwargs=None, max_workgroups=0, static=False, threads=1):
    """Steps the workload on the GPU and the oracle on the blocks; compares after every step.

    shadow=True keeps a second copy of the observed worker's state that is stepped with the
    three single-tensor calls, and requires whole-arena bit equality with the fused state.
    wl_kwargs: forms of the workload (peers in the sparse form, 16-bit gradients, peers' gradients
    resident so that correction passes sum in the kernel); max_workgroups: bounded grids;
    static: the pass goes through cdsgd_step_fused_static instead of the plan.
    threads: the oracle's blocks are stepped by that many host threads (they are independent: the path is
    elementwise; the C oracle runs outside the interpreter lock)."""
    pkg, runner, synth = P
    wl = runner.Workload(cfg, dense=dense, self_rank=self_rank, **(wl_kwargs or {}))
    wl.plan.set_max_workgroups(max_workgroups)
    sh = None
    if shadow:
        sh = dict(w_global=wl.w_global.clone(), w_local=wl.w_local.clone(), residual=wl.residual.clone(),
                  packed_self=wl.packed_self.clone())
    N, t = cfg.num_workers, cfg.threshold
    sims = [oracle.Simulation(wl.view(wl.w_global, i)[a: a + ln].cpu().numpy(), N, cfg.k, t, cfg.lr, cfg.lr,
                              self_rank) for (i, a, ln) in blocks]
    nonzero_codes = 0
    total_codes = 0
    bit_equal = [0, 0]
    for s in range(steps):
        cap = wl.prepare_step(s, capture=blocks)
        comp = wl.compressed(s)
        r_old = wl.residual.clone() if (comp and shadow) else None
        if static:
            pkg.binding.cdsgd_step_fused_static(wl._plan_tensors(), wl._plan_peers(), N, self_rank, s, cfg.k, t,
                                                cfg.lr, cfg.lr)
        elif fused:
            wl.fused_step(s)
        else:
            wl.unfused_step(s)
        torch.cuda.synchronize()
        if shadow:
            # three-call path on the copy, then swap back
            live = dict(w_global=wl.w_global, w_local=wl.w_local, residual=wl.residual, packed_self=wl.packed_self)
            for key in sh:
                setattr(wl, key, sh[key])
            wl.unfused_step(s)
            torch.cuda.synchronize()
            for key in sh:
                setattr(wl, key, live[key])
                assert torch.equal(live[key].view(torch.int32), sh[key].view(torch.int32)), \
                    "fused vs three-call path differ in %s at step %d" % (key, s)
            if comp:
                # conservation over the whole arena: (r_old + g) - value(code) == r_new, in fp32
                by = wl.packed_self.view(torch.uint8)
                a = r_old + wl.grad
                for c4 in range(4):
                    code = (by >> (2 * c4)) & 3
                    assert int((code == 3).sum()) == 0
                    val = torch.where(code == 1, t, 0.0) - torch.where(code == 2, t, 0.0)
                    ok = torch.equal((a[c4::4] - val.to(torch.float32)).view(torch.int32),
                                     wl.residual[c4::4].view(torch.int32))
                    assert ok, "conservation broken at step %d" % s
        def oracle_step(b):
            return sims[b].step([np.ascontiguousarray(cap[j][b]) for j in range(N)])

        if threads > 1:
            with ThreadPoolExecutor(max_workers=threads) as pool:
                stepped = list(pool.map(oracle_step, range(len(blocks))))
        else:
            stepped = [oracle_step(b) for b in range(len(blocks))]
        for b, (i, a, ln) in enumerate(blocks):
            c, agg, words = stepped[b]
            stepped[b] = None
            assert c == comp
            tag = "%s step %d block %d (tensor %d, start %d, len %d)" % (cfg.name, s, b, i, a, ln)
            sl = slice(a, a + ln)
            wsl = slice(a // 16, a // 16 + (ln + 15) // 16)
            if comp:
                got = wl.pview(wl.packed_self, i)[wsl].cpu().numpy()
                assert_bits_equal(got, words[self_rank].view(np.int32), "packed_self " + tag)
                assert_bits_equal(wl.view(wl.residual, i)[sl].cpu().numpy(), sims[b].residual[self_rank],
                                  "residual " + tag)
                codes = oracle.unpack(words[self_rank], ln)
                nonzero_codes += int((codes != 0).sum())
                total_codes += ln
                if check_peers:
                    for j in range(N):
                        if j == self_rank:
                            continue
                        assert_bits_equal(wl.pview(wl.peer_packed[j], i)[wsl].cpu().numpy(),
                                          words[j].view(np.int32), "peer %d packed " % j + tag)
                        assert_bits_equal(wl.view(wl.peer_residual[j], i)[sl].cpu().numpy(),
                                          sims[b].residual[j], "peer %d residual " % j + tag)
            else:
                assert_bits_equal(wl.view(wl.agg_full, i)[sl].cpu().numpy(), agg, "agg_full " + tag)
                assert_bits_equal(wl.view(wl.residual, i)[sl].cpu().numpy(), sims[b].residual[self_rank],
                                  "residual (correction) " + tag)
            gw = wl.view(wl.w_global, i)[sl].cpu().numpy()
            gl = wl.view(wl.w_local, i)[sl].cpu().numpy()
            assert_close(gw, sims[b].w_global, "w_global " + tag)
            assert_close(gl, sims[b].w_local, "w_local " + tag)
            for got, want in ((gw, sims[b].w_global), (gl, sims[b].w_local)):
                e, n = count_bit_equal(got, want)
                bit_equal[0] += e
                bit_equal[1] += n
    wl.destroy()
    # both sides use the same single-rounding form, so bit equality is the expected outcome
    assert bit_equal[0] == bit_equal[1], "weights within 1e-6 but only %d of %d bit-equal" % tuple(bit_equal)
    return nonzero_codes, total_codes


@pytest.mark.parametrize("fused", [True, False], ids=["fused", "threecall"])
@pytest.mark.parametrize("dense", [False, True], ids=["literal", "dense"])
def test_c1_single_tensor_whole_run(P, oracle, dense, fused):
    cfg = P[2].config("c1_single")
    nz, tot = _run(P, oracle, cfg, dense, cfg.iterations, _whole(cfg), fused=fused)
    assert tot == 6 * 65536                 # 6 of the 8 iterations are compressed (k = 4)
    assert nz > (0.2 * tot if dense else 0)  # the literal recipe fires a little, the dense one a lot


@pytest.mark.parametrize("fused", [True, False], ids=["fused", "threecall"])
@pytest.mark.parametrize("dense", [False, True], ids=["literal", "dense"])
def test_c2_resnet20_whole_run(P, oracle, dense, fused):
    cfg = P[2].config("c2_resnet20")
    nz, tot = _run(P, oracle, cfg, dense, cfg.iterations, _whole(cfg), fused=fused)
    assert tot == 15 * cfg.elements
    if dense:
        assert nz > 0.2 * tot


def test_c2_other_worker_positions(P, oracle):
    cfg = P[2].config("c2_resnet20")
    for self_rank in (3, 7):
        _run(P, oracle, cfg, True, 6, _whole(cfg), fused=True, self_rank=self_rank)


@pytest.mark.parametrize("dense", [False, True], ids=["literal", "dense"])
def test_c3_resnet50_full_size_sampled(P, oracle, dense):
    cfg = P[2].config("c3_resnet50")
    rng = np.random.default_rng(33)
    blocks = _sample_blocks(cfg, rng, 24, 1 << 13)
    # the literal recipe runs all 50 iterations (7 correction / 43 compressed), the dense one 20
    nz, tot = _run(P, oracle, cfg, dense, cfg.iterations if not dense else 20, blocks, shadow=True)
    if dense:
        assert nz > 0.2 * tot


@pytest.mark.parametrize("dense", [False, True], ids=["literal", "dense"])
def test_c4_vgg16_full_size_sampled(P, oracle, dense):
    cfg = P[2].config("c4_vgg16")
    rng = np.random.default_rng(44)
    blocks = _sample_blocks(cfg, rng, 20, 1 << 13)
    # the literal recipe runs all 20 iterations (3 correction / 17 compressed), the dense one 10
    nz, tot = _run(P, oracle, cfg, dense, cfg.iterations if not dense else 10, blocks, shadow=True)
    if dense:
        assert nz > 0.2 * tot


def test_c5_flat_bucket_full_size_sampled(P, oracle):
    """4 GiB bucket, t = 0.05 (not a power of two: the literal fp32 chain is what runs)."""
    cfg = P[2].config("c5_flat4g")
    rng = np.random.default_rng(55)
    n = cfg.sizes[0]
    blocks = [(0, 0, 1 << 14), (0, n - (1 << 14), 1 << 14), (0, (1 << 29) - 4096, 8192),   # around 2 GiB
              (0, (1 << 28) * 3 - 4096, 8192)]
    for _ in range(28):
        blocks.append((0, int(rng.integers(0, n // 16 - 1024)) * 16, 1 << 14))
    # all 10 iterations: one correction, nine compressed
    nz, tot = _run(P, oracle, cfg, False, cfg.iterations, blocks, shadow=True)
    # first compressed step fires with probability exp(-2.5); later ones a little more
    assert 0.05 * tot < nz < 0.25 * tot


VARIANTS = {
    "sparse_peers": dict(wl_kwargs=dict(sparse_peers=True), shadow=True),
    "bf16_gradients": dict(wl_kwargs=dict(grad_dtype=torch.bfloat16)),
    "fp16_gradients": dict(wl_kwargs=dict(grad_dtype=torch.float16)),
    "sum_in_kernel": dict(wl_kwargs=dict(full_grads=True), shadow=True),
    "bounded_grid": dict(max_workgroups=1024, shadow=True),
    "no_alloc_entry": dict(static=True, shadow=True),
}


@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_c4_vgg16_full_size_other_forms(P, oracle, variant):
    """The other forms of the pass that the benchmark times on the VGG-16-shaped list, at that size:
    sampled blocks against the oracle after every iteration (two correction passes, eight compressed
    ones, dense recipe), and, where the gradients are fp32, the whole arena against the three
    single-tensor calls."""
    cfg = P[2].config("c4_vgg16")
    rng = np.random.default_rng(4400 + sorted(VARIANTS).index(variant))
    blocks = _sample_blocks(cfg, rng, 12, 1 << 13)
    nz, tot = _run(P, oracle, cfg, True, 10, blocks, **VARIANTS[variant])
    assert nz > 0.2 * tot


@pytest.mark.parametrize("variant", ["no_alloc_entry", "sparse_peers"])
def test_c5_flat_bucket_full_size_other_forms(P, oracle, variant):
    """The 4 GiB bucket (2^30 elements in one tensor, chain form of the decode) through the entry point
    that allocates nothing (262,144 chunks in its static table) and with the peers' streams in the
    sparse form: first, last and random blocks against the oracle, whole arena against the three calls."""
    cfg = P[2].config("c5_flat4g")
    rng = np.random.default_rng(5500 + len(variant))
    n = cfg.sizes[0]
    blocks = [(0, 0, 1 << 14), (0, n - (1 << 14), 1 << 14), (0, (1 << 29) - 4096, 8192)]
    for _ in range(13):
        blocks.append((0, int(rng.integers(0, n // 16 - 1024)) * 16, 1 << 14))
    nz, tot = _run(P, oracle, cfg, False, 4, blocks, **VARIANTS[variant])
    assert 0.05 * tot < nz < 0.25 * tot


@pytest.mark.parametrize("name", ["c3_resnet50", "c4_vgg16"])
def test_whole_list_every_element(P, oracle, name):
    """The ResNet-50- and VGG-16-shaped lists at full size with EVERY element compared with the oracle (not
    sampled blocks): one correction pass and two compressed ones, dense recipe, the oracle stepped by 16
    host threads over 4 Mi-element blocks.  (The played peers' streams are checked on samples by the tests
    above; here only the observed worker's outputs are downloaded.)"""
    cfg = P[2].config(name)
    blocks = _partition(cfg, 1 << 22)
    assert sum(ln for _, _, ln in blocks) == cfg.elements
    nz, tot = _run(P, oracle, cfg, True, 3, blocks, check_peers=False, threads=16)
    assert tot == 2 * cfg.elements and nz > 0.2 * tot


def test_c5_flat_bucket_every_element(P, oracle):
    """The 4 GiB bucket with EVERY one of its 2^30 elements compared with the oracle, for the first two
    iterations: a correction pass, then a compressed pass (the residuals are still zero when it starts, so
    no earlier iteration's state is needed on the host).  All 16 workers' gradients stay resident on the
    GPU; after each pass the buffer is walked in blocks of 4 Mi elements: the workers' gradients of the
    block come down, 16 host threads step the oracle from the weights the pass started with, and the
    block's packed words, residual and both weights are compared bit for bit."""
    pkg, runner, synth = P
    cfg = synth.config("c5_flat4g")
    n, N, t = cfg.sizes[0], cfg.num_workers, cfg.threshold
    wl = runner.Workload(cfg, full_grads=True)
    blen = 1 << 22
    starts = list(range(0, n, blen))
    assert len(starts) * blen == n
    for it in (0, 1):
        w_before = wl.w_global.clone()
        wl.prepare_step(it)
        assert wl.compressed(it) == (it == 1)
        wl.fused_step(it)                    # the correction pass sums the 16 resident gradients in the kernel
        torch.cuda.synchronize()

        def check(a, it=it, w_before=w_before):
            sl, wsl = slice(a, a + blen), slice(a // 16, (a + blen) // 16)
            grads = [(wl.grad if j == 0 else wl.peer_grad[j])[sl].cpu().numpy() for j in range(N)]
            sim = oracle.Simulation(w_before[sl].cpu().numpy(), N, cfg.k, t, cfg.lr, cfg.lr, 0)
            sim.count = it                   # the loop's counter before this pass; residuals are zero either way
            comp, agg, words = sim.step(grads)
            assert comp == (it == 1)
            tag = "iteration %d, block at %d" % (it, a)
            fired = 0
            if comp:
                assert_bits_equal(wl.packed_self[wsl].cpu().numpy(), words[0].view(np.int32), "packed_self " + tag)
                fired = int((oracle.unpack(words[0], blen) != 0).sum())
            assert_bits_equal(wl.residual[sl].cpu().numpy(), sim.residual[0], "residual " + tag)
            assert_bits_equal(wl.w_global[sl].cpu().numpy(), sim.w_global, "w_global " + tag)
            assert_bits_equal(wl.w_local[sl].cpu().numpy(), sim.w_local, "w_local " + tag)
            return fired

        with ThreadPoolExecutor(max_workers=16) as pool:
            fired = sum(pool.map(check, starts))
        if it == 1:
            assert 0.05 * n < fired < 0.15 * n   # exp(-2.5) = 8.2 % of the codes fire on the first compressed pass
        del w_before
    wl.destroy()
