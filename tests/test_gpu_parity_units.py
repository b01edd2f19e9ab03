"""GPU parity, entry point by entry point: HIP library (through the C ABI) vs the CPU oracle,
element by element on the same seeded inputs.  Sizes span several chunks (4096 elements),
several waves, and every kind of ragged tail.  Packed words and residuals: bit-exact.
Aggregate and weights: within 1e-6 relative (bit equality is also counted and required
where both sides use the same single-rounding form)."""
import numpy as np
import pytest
import torch

from helpers import assert_bits_equal, assert_close

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 3, 4, 5, 15, 16, 17, 31, 33, 63, 64, 65, 255, 1023, 1024, 1025, 4093, 4095, 4096,
         4097, 4111, 8191, 12289, 16384, 65536, 100003]
GUARD = 64  # sentinel elements on both sides of every output buffer


@pytest.fixture(scope="module")
def B():
    from paper_2106_10796_amd import binding, build
    build.ensure_built()
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def guarded(n, dtype, fill):
    """A device buffer with sentinels around an aligned interior view."""
    full = torch.full((n + 2 * GUARD,), fill, dtype=dtype, device="cuda")
    return full, full[GUARD: GUARD + n]


def guards_intact(full, n, fill):
    f = full.cpu()
    return bool((f[:GUARD] == fill).all() and (f[GUARD + n:] == fill).all())


def rand_inputs(rng, n, t):
    g = (rng.normal(0, 1.2 * t, n)).astype(np.float32)
    r = rng.uniform(-t, t, n).astype(np.float32)
    # force exact-threshold cases in
    if n >= 4:
        r[0], g[0] = 0.0, t
        r[1], g[1] = 0.0, -t
        r[2], g[2] = np.float32(t) / 2, np.float32(t) / 2
        r[3], g[3] = 0.0, np.nextafter(np.float32(t), np.float32(0))
    return g, r


@pytest.mark.parametrize("t", [0.5, 0.05])
@pytest.mark.parametrize("n", SIZES)
def test_quantize_pack(B, oracle, n, t):
    rng = np.random.default_rng(1000 + n)
    g, r = rand_inputs(rng, n, t)
    nw = B.packed_words(n)
    dg = torch.from_numpy(g).cuda()
    rfull, dr = guarded(n, torch.float32, 7.0)
    dr.copy_(torch.from_numpy(r))
    pfull, dp = guarded(nw, torch.int32, -1)     # stale 0xFFFFFFFF: pad bits must be cleared
    B.cdsgd_quantize_pack(dg, dr, dp, t)
    torch.cuda.synchronize()
    r_o = r.copy()
    words = oracle.quantize_pack(g, r_o, t)
    assert_bits_equal(dp.cpu().numpy(), words.view(np.int32), "packed n=%d" % n)
    assert_bits_equal(dr.cpu().numpy(), r_o, "residual n=%d" % n)
    assert guards_intact(rfull, n, 7.0) and guards_intact(pfull, nw, -1)
    assert_bits_equal(dg.cpu().numpy(), g, "grad must not be written")


def test_quantize_pack_special_values(B, oracle):
    den = np.float32(1e-45)
    g = np.array([np.nan, np.inf, -np.inf, den, -den, 0.0, -0.0, 3e-39, 1e30, -1e30], np.float32)
    r = np.array([0, 0, 0, den, 0, 0, -0.0, 3e-39, 1e30, 0.25], np.float32)
    dg, dr = torch.from_numpy(g).cuda(), torch.from_numpy(r).cuda()
    dp = B.new_packed(g.size)
    B.cdsgd_quantize_pack(dg, dr, dp, 0.5)
    r_o = r.copy()
    words = oracle.quantize_pack(g, r_o, 0.5)
    assert_bits_equal(dp.cpu().numpy(), words.view(np.int32), "packed")
    assert_bits_equal(dr.cpu().numpy(), r_o, "residual (NaN matches NaN)")
    out = dr.cpu().numpy()
    assert out[3] == np.float32(3e-45) and out[7] != 0.0   # denormals survive, no flush


@pytest.mark.parametrize("t", [0.5, 0.05, 0.3, 2.0 ** -20])
@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 8, 9, 12, 13, 16, 17, 33, 64])
def test_decode_sum(B, oracle, N, t):
    rng = np.random.default_rng(2000 + N)
    for n in (1, 17, 4095, 4097, 20000):
        nw = B.packed_words(n)
        # codes with a bias towards one sign so that sums run up, the unused code 3 included,
        # and random garbage in the pad bits of the last word (must not matter)
        codes = rng.choice(4, size=(N, n), p=[0.3, 0.4, 0.25, 0.05]).astype(np.uint8)
        words = [oracle.pack(np.ascontiguousarray(codes[j])) for j in range(N)]
        if n % 16:
            for w in words:
                w[-1] |= np.uint32(rng.integers(0, 1 << 32) & ~((1 << (2 * (n % 16))) - 1) & 0xFFFFFFFF)
        dw = [torch.from_numpy(w.view(np.int32)).cuda() for w in words]
        afull, da = guarded(n, torch.float32, 9.0)
        B.cdsgd_decode_sum(dw, da, t)
        torch.cuda.synchronize()
        agg = oracle.decode_sum(words, n, t)
        assert_close(da.cpu().numpy(), agg, "agg N=%d n=%d t=%g" % (N, n, t))
        assert_bits_equal(da.cpu().numpy(), agg, "agg bits N=%d n=%d t=%g" % (N, n, t))
        assert guards_intact(afull, n, 9.0)


@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4096, 4099, 70001])
@pytest.mark.parametrize("mode", ["both", "local", "global"])
def test_update(B, oracle, n, mode):
    rng = np.random.default_rng(3000 + n)
    W = rng.normal(0, 1, n).astype(np.float32)
    g = rng.normal(0, 1, n).astype(np.float32)
    agg = (rng.integers(-16, 17, n) * 0.5).astype(np.float32)
    N, lr_l, lr_g = 3, 0.4, 0.1
    wfull, dW = guarded(n, torch.float32, 5.0)
    dW.copy_(torch.from_numpy(W))
    lfull, dL = guarded(n, torch.float32, 6.0)
    dg, da = torch.from_numpy(g).cuda(), torch.from_numpy(agg).cuda()
    W_o, L_o = W.copy(), np.full(n, 6.0, np.float32)
    if mode == "both":
        B.cdsgd_update(dW, dL, dg, da, lr_l, lr_g, N)
        oracle.update(W_o, L_o, g, agg, lr_l, lr_g, N)
    elif mode == "local":
        B.cdsgd_update(dW, dL, dg, None, lr_l, lr_g, N)
        oracle.update(W_o, L_o, g, None, lr_l, lr_g, N)
    else:
        B.cdsgd_update(dW, None, None, da, lr_l, lr_g, N)
        oracle.update(W_o, None, None, agg, lr_l, lr_g, N)
    torch.cuda.synchronize()
    assert_close(dW.cpu().numpy(), W_o, "w_global")
    assert_close(dL.cpu().numpy(), L_o, "w_local")
    assert_bits_equal(dW.cpu().numpy(), W_o, "w_global bits")
    assert_bits_equal(dL.cpu().numpy(), L_o, "w_local bits")
    assert guards_intact(wfull, n, 5.0) and guards_intact(lfull, n, 6.0)


def test_probe_streams_moves_what_it_says(B):
    """The measurement aid: every write stream receives the sum of the read streams plus its index,
    nothing outside the buffers is touched, a read-only run writes nothing."""
    rng = np.random.default_rng(3500)
    n = 256 * 37
    reads = [torch.from_numpy(rng.normal(0, 1, n).astype(np.float32)).cuda() for _ in range(17)]
    for R in (0, 1, 2, 3, 4, 9, 17):
        for W in range(0, 4):
            if R + W == 0:
                continue
            fulls = [guarded(n, torch.float32, 4.0) for _ in range(W)]
            sink = torch.full((n // 256,), 7.0, device="cuda")
            B.cdsgd_probe_streams(reads[:R], [v for _, v in fulls], sink, lds_bytes=(0, 8192, 16384)[(R + W) % 3])
            torch.cuda.synchronize()
            want = np.zeros(n, np.float32)
            for i in range(R):
                want = want + reads[i].cpu().numpy()              # same order of adds as the kernel
            for i, (full, v) in enumerate(fulls):
                assert_bits_equal(v.cpu().numpy(), (want + np.float32(i)).astype(np.float32), "probe R=%d W=%d stream %d" % (R, W, i))
                assert guards_intact(full, n, 4.0)
            assert bool((sink == 7.0).all())


def _run_layer_list(B, oracle, sizes, N, self_rank, k, t, steps, seed, lr_l=0.4, lr_g=0.1, stepper=None):
    """Fused step vs oracle vs the three-call composition on an arbitrary layer list.
    stepper(plan, s): how iteration s is enqueued (default: one cdsgd_step_fused over the list); the plan
    carries what a stepper may need beyond it as attributes (layer_list, peer_rows)."""
    rng = np.random.default_rng(seed)
    T = len(sizes)
    dev = dict(device="cuda")
    W0 = [rng.normal(0, 0.3, n).astype(np.float32) for n in sizes]
    # two device copies of the state: one stepped by the fused call, one by the three calls
    state = []
    for tag in ("fused", "composed"):
        st = dict(
            w_global=[torch.from_numpy(w).cuda() for w in W0],
            w_local=[torch.zeros(n, dtype=torch.float32, **dev) for n in sizes],
            residual=[torch.zeros(n, dtype=torch.float32, **dev) for n in sizes],
            grad=[torch.zeros(n, dtype=torch.float32, **dev) for n in sizes],
            packed_self=[torch.full((B.packed_words(n),), -1, dtype=torch.int32, **dev) for n in sizes],
            agg_full=[torch.zeros(n, dtype=torch.float32, **dev) for n in sizes],
        )
        state.append(st)
    peers = [None if j == self_rank else [B.new_packed(n) for n in sizes] for j in range(N)]
    tensors = [{key: state[0][key][i] for key in state[0]} for i in range(T)]
    plan = B.Plan(tensors, peers if N > 1 else None, N, self_rank)
    plan.layer_list, plan.peer_rows = tensors, (peers if N > 1 else None)
    sims = [oracle.Simulation(W0[i], N, k, t, lr_l, lr_g, self_rank) for i in range(T)]
    agg_dev = [torch.zeros(n, dtype=torch.float32, **dev) for n in sizes]
    for s in range(steps):
        comp_expected = (s % k) != 0
        for i, n in enumerate(sizes):
            grads = [rng.normal(0, 1.1 * t, n).astype(np.float32) for _ in range(N)]
            comp, agg, words = sims[i].step(grads)
            assert comp == comp_expected
            for st in state:
                st["grad"][i].copy_(torch.from_numpy(grads[self_rank]))
                if not comp:
                    st["agg_full"][i].copy_(torch.from_numpy(agg))
            if comp:
                for j in range(N):
                    if j != self_rank:
                        peers[j][i].copy_(torch.from_numpy(words[j].view(np.int32)))
            sims[i]._last = (comp, agg, words)
        resid_before = [r.clone() for r in state[0]["residual"]]
        packed_before = [p.clone() for p in state[0]["packed_self"]]
        if stepper is None:
            plan.step(s, k, t, lr_l, lr_g)
        else:
            stepper(plan, s)
        # composition on the second copy
        c = state[1]
        for i in range(T):
            if comp_expected:
                B.cdsgd_quantize_pack(c["grad"][i], c["residual"][i], c["packed_self"][i], t)
                streams = [c["packed_self"][i] if j == self_rank else peers[j][i] for j in range(N)]
                B.cdsgd_decode_sum(streams, agg_dev[i], t)
                B.cdsgd_update(c["w_global"][i], c["w_local"][i], c["grad"][i], agg_dev[i], lr_l, lr_g, N)
            else:
                B.cdsgd_update(c["w_global"][i], c["w_local"][i], c["grad"][i], c["agg_full"][i], lr_l, lr_g, N)
        torch.cuda.synchronize()
        f = state[0]
        for i in range(T):
            comp, agg, words = sims[i]._last
            tag = "step %d tensor %d (n=%d)" % (s, i, sizes[i])
            if comp:
                assert_bits_equal(f["packed_self"][i].cpu().numpy(), words[self_rank].view(np.int32), "packed " + tag)
                assert_bits_equal(f["residual"][i].cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
                assert_close(agg_dev[i].cpu().numpy(), agg, "agg " + tag)
            else:
                assert torch.equal(f["residual"][i], resid_before[i]), "residual touched on correction " + tag
                assert torch.equal(f["packed_self"][i], packed_before[i]), "packed touched on correction " + tag
            assert_close(f["w_global"][i].cpu().numpy(), sims[i].w_global, "w_global " + tag)
            assert_close(f["w_local"][i].cpu().numpy(), sims[i].w_local, "w_local " + tag)
            assert_bits_equal(f["w_global"][i].cpu().numpy(), sims[i].w_global, "w_global bits " + tag)
            assert_bits_equal(f["w_local"][i].cpu().numpy(), sims[i].w_local, "w_local bits " + tag)
            # fused == composition of the three calls, bit for bit
            for key in ("w_global", "w_local", "residual", "packed_self"):
                assert torch.equal(f[key][i].view(torch.int32), c[key][i].view(torch.int32)), key + " fused vs composed " + tag
    plan.destroy()


RAGGED = [1, 10, 16, 17, 64, 100, 1000, 4095, 4096, 4097, 9000, 36864, 5, 20011]


@pytest.mark.parametrize("N,t,split", [(4, 0.5, False), (16, 0.05, False), (9, 0.25, True), (2, 0.3, True)])
def test_layer_by_layer_equals_whole_list(B, oracle, N, t, split):
    """The list stepped in ranges, last layers first as back-propagation delivers them, in groups of
    uneven size (Sec. 3.2.2): oracle, three-call composition and untouched outputs as for the whole list."""
    k, lr_l, lr_g = 3, 0.4, 0.1
    T = len(RAGGED)
    cuts = [T, 13, 12, 8, 7, 3, 0]                   # groups [13,14) [12,13) [8,12) [7,8) [3,7) [0,3)

    def stepper(plan, s):
        for hi, lo in zip(cuts[:-1], cuts[1:]):
            if split:
                plan.step_local_range(lo, hi - lo, lr_l)
                plan.step_global_range(lo, hi - lo, s, k, t, lr_g)
            else:
                plan.step_range(lo, hi - lo, s, k, t, lr_l, lr_g)

    _run_layer_list(B, oracle, RAGGED, N, N // 2, k, t, 5, 3600 + N, lr_l, lr_g, stepper=stepper)


def test_a_range_touches_only_its_tensors(B):
    sizes = [5000, 17, 4096, 9000, 300]
    rng = np.random.default_rng(3700)
    dev = dict(device="cuda")
    N, self_rank = 3, 1
    keys = ("w_global", "w_local", "residual", "packed_self")
    st = dict(w_global=[torch.from_numpy(rng.normal(0, 0.3, n).astype(np.float32)).cuda() for n in sizes],
              w_local=[torch.full((n,), 9.0, **dev) for n in sizes],
              residual=[torch.from_numpy(rng.normal(0, 0.3, n).astype(np.float32)).cuda() for n in sizes],
              grad=[torch.from_numpy(rng.normal(0, 0.5, n).astype(np.float32)).cuda() for n in sizes],
              packed_self=[torch.full((B.packed_words(n),), -1, dtype=torch.int32, **dev) for n in sizes],
              agg_full=[torch.from_numpy(rng.normal(0, 0.5, n).astype(np.float32)).cuda() for n in sizes])
    peers = [None if j == self_rank else
             [torch.from_numpy(rng.integers(0, 2**32, B.packed_words(n), dtype=np.uint32).view(np.int32)).cuda()
              for n in sizes] for j in range(N)]
    plan = B.Plan([{key: st[key][i] for key in st} for i in range(len(sizes))], peers, N, self_rank)
    for step in (1, 0):                                # a compressed pass, then a correction pass
        before = {key: [v.clone() for v in st[key]] for key in keys}
        plan.step_range(1, 3, step, 2, 0.5, 0.4, 0.1)
        torch.cuda.synchronize()
        for i in range(len(sizes)):
            inside = 1 <= i < 4
            for key in keys:
                same = torch.equal(st[key][i].view(torch.int32), before[key][i].view(torch.int32))
                if not inside:
                    assert same, "%s of tensor %d outside the range was written (step %d)" % (key, i, step)
                elif key in ("w_global", "w_local"):
                    assert not same, "%s of tensor %d inside the range was not stepped (step %d)" % (key, i, step)
    for first, count in ((-1, 2), (0, 0), (3, 3), (5, 1), (0, 6)):
        with pytest.raises(RuntimeError):
            plan.step_range(first, count, 1, 2, 0.5, 0.4, 0.1)
        with pytest.raises(RuntimeError):
            plan.step_local_range(first, count, 0.4)
        with pytest.raises(RuntimeError):
            plan.step_global_range(first, count, 1, 2, 0.5, 0.1)
    plan.step_range(0, 5, 1, 2, 0.5, 0.4, 0.1)         # the whole list as one range is fine
    torch.cuda.synchronize()
    plan.destroy()


@pytest.mark.parametrize("t", [0.5, 0.05])
@pytest.mark.parametrize("N,self_rank", [(1, 0), (2, 0), (2, 1), (4, 0), (5, 2), (8, 7), (16, 0), (16, 9), (17, 16)])
def test_fused_step_layer_list(B, oracle, N, self_rank, t):
    _run_layer_list(B, oracle, RAGGED, N, self_rank, k=3, t=t, steps=5, seed=4000 + 17 * N + self_rank)


def test_fused_step_max_workers(B, oracle):
    _run_layer_list(B, oracle, [4100, 33], 64, 31, k=4, t=0.05, steps=3, seed=4999)
    _run_layer_list(B, oracle, [4100, 33], 64, 63, k=4, t=0.25, steps=3, seed=4998)


def test_tensor_beyond_2_to_32_elements(B, oracle):
    """One tensor of 2^32 + 4099 elements (17 GB per fp32 buffer): element and byte offsets
    beyond 32 bits, over a million chunks, ragged end.  All three single-tensor calls and the
    fused step, compared with the oracle on blocks at the start, around element 2^31, around
    element 2^32 and at the ragged end (the path is elementwise)."""
    n = (1 << 32) + 4099
    N, self_rank, t, lr_l, lr_g, k = 3, 1, 0.05, 0.4, 0.1, 4
    free, _ = torch.cuda.mem_get_info()
    if free < 130 * (1 << 30):
        pytest.skip("needs about 130 GiB of free HBM")
    nw = B.packed_words(n)
    blocks = [(0, 8192), ((1 << 31) - 4096, 8192), ((1 << 32) - 8192, 8192 + 4099)]

    def take(x, words=False):
        return [x[(a // 16 if words else a): (a // 16 + (ln + 15) // 16) if words else a + ln].cpu().numpy()
                for a, ln in blocks]

    def gauss(seed, std):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        return torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, std, generator=gen)

    # peers' packed streams (their residuals start at zero) via the library itself
    peers, peer_g = [], []
    for j in range(N):
        if j == self_rank:
            peers.append(None)
            peer_g.append(None)
            continue
        g = gauss(900 + j, 0.06)
        r = torch.zeros(n, dtype=torch.float32, device="cuda")
        p = torch.full((nw,), -1, dtype=torch.int32, device="cuda")
        B.cdsgd_quantize_pack(g, r, p, t)
        torch.cuda.synchronize()
        peer_g.append(take(g))
        # standalone quantize_pack against the oracle on the blocks
        for b, (a, ln) in enumerate(blocks):
            r_o = np.zeros(ln, np.float32)
            words = oracle.quantize_pack(peer_g[j][b], r_o, t)
            assert_bits_equal(take(p, True)[b], words.view(np.int32), "peer %d packed block %d" % (j, b))
            assert_bits_equal(take(r)[b], r_o, "peer %d residual block %d" % (j, b))
        peers.append(p)
        del g, r
    g = gauss(901 + self_rank * 7, 0.06)
    W = gauss(777, 0.3)
    Wloc = torch.zeros(n, dtype=torch.float32, device="cuda")
    r = torch.zeros(n, dtype=torch.float32, device="cuda")
    pself = torch.full((nw,), -1, dtype=torch.int32, device="cuda")
    g_b, W_b = take(g), take(W)
    plan = B.Plan([dict(w_global=W, w_local=Wloc, residual=r, grad=g, packed_self=pself)],
                  [[p] if p is not None else None for p in peers], N, self_rank)
    plan.step(1, k, t, lr_l, lr_g)       # a compressed step
    torch.cuda.synchronize()
    # decode_sum and update standalone on the same inputs (W is already updated, so use copies of blocks only)
    agg = torch.empty(n, dtype=torch.float32, device="cuda")
    B.cdsgd_decode_sum([pself if j == self_rank else peers[j] for j in range(N)], agg, t)
    torch.cuda.synchronize()
    got = dict(p=take(pself, True), r=take(r), W=take(W), L=take(Wloc), agg=take(agg))
    for b, (a, ln) in enumerate(blocks):
        sim = oracle.Simulation(W_b[b], N, k, t, lr_l, lr_g, self_rank)
        sim.count = 1
        grads = [g_b[b] if j == self_rank else peer_g[j][b] for j in range(N)]
        comp, agg_o, words = sim.step(grads)
        assert comp
        tag = "block %d (start %d)" % (b, a)
        assert_bits_equal(got["p"][b], words[self_rank].view(np.int32), "packed_self " + tag)
        assert_bits_equal(got["r"][b], sim.residual[self_rank], "residual " + tag)
        assert_close(got["agg"][b], agg_o, "agg " + tag)
        assert_bits_equal(got["agg"][b], agg_o, "agg bits " + tag)
        assert_close(got["W"][b], sim.w_global, "w_global " + tag)
        assert_close(got["L"][b], sim.w_local, "w_local " + tag)
        assert_bits_equal(got["W"][b], sim.w_global, "w_global bits " + tag)
        assert_bits_equal(got["L"][b], sim.w_local, "w_local bits " + tag)
    # the last packed word's unused bits are zero
    assert int(pself[-1].item()) >> (2 * (n % 16)) == 0
    plan.destroy()


def test_fused_step_many_tiny_tensors(B, oracle):
    """1500 tensors of 1..300 elements in one launch (a chunk table of 1500 tail chunks)."""
    rng = np.random.default_rng(77)
    sizes = [int(x) for x in rng.integers(1, 301, 1500)]
    _run_layer_list(B, oracle, sizes, 4, 2, k=2, t=0.5, steps=3, seed=5100)


def test_fused_step_random_configurations(B, oracle):
    """Seeded random layer lists, worker counts, positions, periods and thresholds (both decode
    forms), each checked step by step against the oracle and the three-call composition; every
    third case steps the list as ranges of tensors in a random order, every third through
    cdsgd_step_fused_static.
    CDSGD_FUZZ_CASES raises the number of cases for a longer soak."""
    import os
    cases = int(os.environ.get("CDSGD_FUZZ_CASES", "40"))
    rng = np.random.default_rng(20261127)
    for case in range(cases):
        T = int(rng.integers(1, 9))
        kinds = rng.integers(0, 4, T)
        sizes = []
        for kind in kinds:
            if kind == 0:
                sizes.append(int(rng.integers(1, 70)))                       # tiny, every tail shape
            elif kind == 1:
                sizes.append(int(rng.integers(1, 5)) * 4096 + int(rng.integers(-3, 4)))   # around chunk edges
            elif kind == 2:
                sizes.append(int(rng.integers(70, 20000)))
            else:
                sizes.append(int(rng.integers(1, 40)) * 1024)
        N = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33]))
        self_rank = int(rng.integers(0, N))
        k = int(rng.integers(1, 5))
        t = float(rng.choice([0.5, 0.25, 2.0, 0.05, 0.3, 1e-3, 0.0625, 7.0]))
        stepper, groups = None, None
        if case % 3 == 2:
            # every third case enqueues the list as ranges: a random partition, in a random order
            r2 = np.random.default_rng(5150 + case)
            cuts = sorted(set([0, T] + [int(x) for x in r2.integers(0, T + 1, int(r2.integers(0, 4)))]))
            groups = [(lo, hi - lo) for lo, hi in zip(cuts[:-1], cuts[1:])]
            groups = [groups[i] for i in r2.permutation(len(groups))]

            def stepper(plan, s, groups=groups, k=k, t=t):
                for lo, cnt in groups:
                    plan.step_range(lo, cnt, s, k, t, 0.4, 0.1)
        elif case % 3 == 1:
            # ... and every third one goes through the entry point that allocates nothing
            def stepper(plan, s, N=N, self_rank=self_rank, k=k, t=t):
                B.cdsgd_step_fused_static(plan.layer_list, plan.peer_rows, N, self_rank, s, k, t, 0.4, 0.1)
        try:
            _run_layer_list(B, oracle, sizes, N, self_rank, k=k, t=t, steps=int(rng.integers(2, 5)),
                            seed=9000 + case, stepper=stepper)
        except AssertionError as e:
            raise AssertionError("case %d: sizes=%s N=%d self=%d k=%d t=%g ranges=%s: %s"
                                 % (case, sizes, N, self_rank, k, t, groups, e))
        if cases > 100 and case % 100 == 99:
            print("fuzz: %d cases done" % (case + 1), flush=True)
