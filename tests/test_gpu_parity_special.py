"""GPU parity on the values random data never holds: NaN, +-Inf, denormals, -0, exact +-t and the
largest finite numbers, sent through every fused kernel (compressed passes with both decode
forms, correction and warm-up passes with both aggregate sources, interior and tail chunks),
and every one of the 65,536 bit patterns of fp16 and of bf16 through the typed plans.
Everything is compared with the oracle bit for bit (any NaN matches any NaN)."""
import numpy as np
import pytest
import torch

from helpers import assert_bits_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2106_10796_amd import binding, build
    build.ensure_built()
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _specials(t):
    t = np.float32(t)
    den = np.float32(1e-45)
    big = np.finfo(np.float32).max
    up = np.nextafter(t, np.float32(np.inf))
    dn = np.nextafter(t, np.float32(0))
    return np.array([np.nan, np.inf, -np.inf, den, -den, 0.0, -0.0, 3e-39, -3e-39, big, -big, t, -t, up, -up,
                     dn, -dn, 2 * t, -2 * t, 1e30, -1e30, t / 2, -t / 2, 1.17549435e-38], np.float32)


def _sprinkle(rng, a, t, where):
    """Overwrite a[where[i]] with special values, cycling through the list in a seeded order."""
    sp = _specials(t)
    a[where] = sp[rng.permutation(len(where)) % sp.size]
    return a


def _positions(n):
    """Element positions in an n-element tensor: its start, around every 4096-element chunk edge,
    and the whole ragged end (the last partial quad and the quads before it)."""
    pos = set(range(min(n, 8)))
    for edge in range(4096, n, 4096):
        pos.update(range(edge - 4, min(n, edge + 4)))
    pos.update(range(max(0, n - 11), n))
    pos.update(range(17, n, 97))
    return np.array(sorted(pos), np.int64)


SIZES = [2 * 4096 + 5, 13, 4096, 3, 4096 + 1022]


@pytest.mark.parametrize("full_grads", [True, False], ids=["kernel_sum", "agg_full"])
@pytest.mark.parametrize("t", [0.5, 0.05], ids=["count_form", "chain_form"])
def test_special_values_through_every_fused_pass(B, oracle, t, full_grads):
    """Alg. 1 with one warm-up step, then two periods of k = 3: warm-up passes (copy and local
    rule), correction passes and compressed passes, special values in the gradients of every
    worker, in the residuals and in the weights."""
    rng = np.random.default_rng(515 + int(1000 * t) + full_grads)
    N, self_rank, k, warmup_n, lr_l, lr_g = 4, 1, 3, 1, 0.4, 0.1
    T = len(SIZES)
    W0 = [_sprinkle(rng, rng.normal(0, 0.3, n).astype(np.float32), t, _positions(n)[::3]) for n in SIZES]
    R0 = [[_sprinkle(rng, rng.uniform(-t, t, n).astype(np.float32), t, _positions(n)[j % 3::3]) for n in SIZES]
          for j in range(N)]
    # one element is kept denormal on purpose: residual 3e-39, own gradient 1e-45 on every pass
    DEN_POS = 5
    R0[self_rank][0][DEN_POS] = np.float32(3e-39)
    dev = dict(device="cuda")
    st = dict(w_global=[torch.from_numpy(w).cuda() for w in W0],
              w_local=[torch.full((n,), -9.0, **dev) for n in SIZES],
              residual=[torch.from_numpy(r).cuda() for r in R0[self_rank]],
              grad=[torch.zeros(n, **dev) for n in SIZES],
              packed_self=[torch.full((B.packed_words(n),), -1, dtype=torch.int32, **dev) for n in SIZES],
              agg_full=[torch.zeros(n, **dev) for n in SIZES])
    peers = [None if j == self_rank else [B.new_packed(n) for n in SIZES] for j in range(N)]
    peer_g = [None if j == self_rank else [torch.zeros(n, **dev) for n in SIZES] for j in range(N)]
    plan = B.Plan([{key: st[key][i] for key in st} for i in range(T)], peers, N, self_rank)
    if full_grads:
        plan.bind_full_grads(peer_g)
    trainer = B.Trainer(plan, warmup_n, k, t, lr_l, lr_g)
    sims = []
    for i, n in enumerate(SIZES):
        sim = oracle.TrainerSimulation(W0[i], N, warmup_n, k, t, lr_l, lr_g, self_rank,
                                       w_local0=np.full(n, -9.0, np.float32))
        for j in range(N):
            sim.residual[j][:] = R0[j][i]
        sims.append(sim)
    saw_nan_code = False
    for it in range(warmup_n + 1 + 2 * k):
        outs = []
        for i, n in enumerate(SIZES):
            grads = [_sprinkle(rng, rng.normal(0, 1.1 * t, n).astype(np.float32), t, _positions(n)[(it + j) % 2::2])
                     for j in range(N)]
            if i == 0:
                grads[self_rank][DEN_POS] = np.float32(1e-45)
            mode, agg, words = sims[i].step(grads)
            outs.append((mode, words))
            st["grad"][i].copy_(torch.from_numpy(grads[self_rank]))
            for j in range(N):
                if j == self_rank:
                    continue
                if mode == 1:
                    peers[j][i].copy_(torch.from_numpy(words[j].view(np.int32)))
                elif full_grads:
                    peer_g[j][i].copy_(torch.from_numpy(grads[j]))
            if mode != 1 and not full_grads:
                st["agg_full"][i].copy_(torch.from_numpy(agg))
        kind = trainer.step()
        torch.cuda.synchronize()
        for i, n in enumerate(SIZES):
            mode, words = outs[i]
            assert mode == kind
            tag = "t=%g iteration %d (mode %d) tensor %d (n=%d)" % (t, it, mode, i, n)
            if mode == 1:
                assert_bits_equal(st["packed_self"][i].cpu().numpy(), words[self_rank].view(np.int32), "packed " + tag)
            assert_bits_equal(st["residual"][i].cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
            assert_bits_equal(st["w_global"][i].cpu().numpy(), sims[i].w_global, "w_global " + tag)
            assert_bits_equal(st["w_local"][i].cpu().numpy(), sims[i].w_local, "w_local " + tag)
            saw_nan_code = saw_nan_code or bool(np.isnan(sims[i].residual[self_rank]).any())
    # the special values really went through: NaN residuals exist, and the denormal element took
    # its 2 (k - 1) denormal increments without being flushed
    assert saw_nan_code
    want = np.float32(3e-39)
    for _ in range(2 * (k - 1)):
        want = np.float32(want + np.float32(1e-45))
    got = st["residual"][0].cpu().numpy()[DEN_POS]
    assert got == want and got != np.float32(3e-39) and abs(got) < np.float32(1.17549435e-38)
    trainer.destroy()
    plan.destroy()


def _all_patterns(kind):
    """(fp32 values, torch tensor of the 16-bit type) for all 65,536 bit patterns, in bit order."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    if kind == "float16":
        wide = bits.view(np.float16).astype(np.float32)          # exact: every fp16 is an fp32
        dt = torch.float16
    else:
        wide = (bits.astype(np.uint32) << 16).view(np.float32)   # bf16 is the upper half of an fp32
        dt = torch.bfloat16
    return bits, wide, dt


def _as_dev16(bits, dt):
    return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(dt)


@pytest.mark.parametrize("kind", ["float16", "bfloat16"])
def test_every_16_bit_pattern_widens_exactly(B, oracle, kind):
    """A layer list that holds every fp16 (bf16) bit pattern as the own gradient, in interior
    chunks, in tail chunks and in tensors of 1 to 3 elements (the scalar loads of a partial
    quad); the peers' gradients hold the same patterns in another order.  One correction pass
    (kernel sum: the peers' 16-bit gradients are widened too), then compressed passes with both
    decode forms; the oracle gets numpy's exact widening."""
    bits, wide, dt = _all_patterns(kind)
    rng = np.random.default_rng(616)
    # sizes: two with tails, then 300 tiny tensors that repeat the most delicate patterns
    delicate = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF, 0x7C00, 0xFC00, 0x7C01,
                         0x7E00, 0xFE00, 0x7FFF, 0xFFFF, 0x3800, 0xB800, 0x007F, 0x0080, 0x7F80, 0xFF80, 0x7F7F,
                         0x7FC0, 0x3F00, 0xBF00, 0x2A66], np.uint16)
    sizes = [4099, 65536 - 4099]
    own_bits = [bits[:4099], bits[4099:]]
    tiny_rng = np.random.default_rng(617)
    for _ in range(300):
        n = int(tiny_rng.integers(1, 4))
        sizes.append(n)
        own_bits.append(delicate[tiny_rng.integers(0, delicate.size, n)])
    T = len(sizes)
    N, self_rank, k, lr_l, lr_g = 3, 2, 4, 0.4, 0.1

    def widen(b):
        return wide[b.astype(np.int64)]

    peer_bits = [[np.ascontiguousarray(np.roll(b[::-1], 7 * (j + 1))) for b in own_bits] for j in range(N)]
    peer_bits[self_rank] = own_bits
    for t in (0.5, 0.05):
        dev = dict(device="cuda")
        W0 = [rng.normal(0, 0.3, n).astype(np.float32) for n in sizes]
        st = dict(w_global=[torch.from_numpy(w).cuda() for w in W0],
                  w_local=[torch.zeros(n, **dev) for n in sizes],
                  residual=[torch.zeros(n, **dev) for n in sizes],
                  grad=[_as_dev16(b, dt) for b in own_bits],
                  packed_self=[torch.full((B.packed_words(n),), -1, dtype=torch.int32, **dev) for n in sizes])
        peers = [None if j == self_rank else [B.new_packed(n) for n in sizes] for j in range(N)]
        peer_g = [None if j == self_rank else [_as_dev16(b, dt) for b in peer_bits[j]] for j in range(N)]
        plan = B.Plan([{key: st[key][i] for key in st} for i in range(T)], peers, N, self_rank, grad_dtype=dt)
        plan.bind_full_grads(peer_g)
        sims = [oracle.Simulation(W0[i], N, k, t, lr_l, lr_g, self_rank) for i in range(T)]
        for s in range(3):          # correction, compressed, compressed (residuals carry over)
            outs = []
            for i in range(T):
                comp, agg, words = sims[i].step([widen(peer_bits[j][i]) for j in range(N)])
                outs.append((comp, words))
                if comp:
                    for j in range(N):
                        if j != self_rank:
                            peers[j][i].copy_(torch.from_numpy(words[j].view(np.int32)))
            plan.step(s, k, t, lr_l, lr_g)
            torch.cuda.synchronize()
            for i in range(T):
                comp, words = outs[i]
                tag = "%s t=%g step %d tensor %d (n=%d)" % (kind, t, s, i, sizes[i])
                if comp:
                    assert_bits_equal(st["packed_self"][i].cpu().numpy(), words[self_rank].view(np.int32), "packed " + tag)
                assert_bits_equal(st["residual"][i].cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
                assert_bits_equal(st["w_global"][i].cpu().numpy(), sims[i].w_global, "w_global " + tag)
                assert_bits_equal(st["w_local"][i].cpu().numpy(), sims[i].w_local, "w_local " + tag)
        plan.destroy()
    # direct check of the widening, independent of the quantiser's decisions: with a threshold no
    # finite 16-bit value reaches, one compressed pass from a zero residual leaves residual == widened g
    # (a residual of -0 makes residual + g reproduce g bit for bit, signed zeros included)
    t_big = float(2.0 ** 100) if kind == "bfloat16" else 131072.0
    finite_small = ~(np.abs(wide) >= np.float32(t_big))          # NaN patterns stay in: NaN must come out as NaN
    g16 = _as_dev16(bits, dt)
    res = torch.full((65536,), -0.0, device="cuda")
    loc = torch.zeros(65536, device="cuda")
    wg = torch.zeros(65536, device="cuda")
    plan = B.Plan([dict(w_global=wg, w_local=loc, residual=res, grad=g16, packed_self=B.new_packed(65536))],
                  None, 1, 0, grad_dtype=dt)
    plan.step(1, 4, t_big, 1.0, 1.0)
    torch.cuda.synchronize()
    got = res.cpu().numpy()
    assert_bits_equal(got[finite_small], wide[finite_small], "%s widened values" % kind)
    assert np.isnan(got[np.isnan(wide)]).all()
    plan.destroy()
